// Host side of libhxt: launch logic, accumulator bookkeeping, staging copies, the micro-batch
// stream, and the C ABI declared in include/hxt.h.  The kernels are in hxt_kernels.h, the
// planner (pure host, no HIP) in hxt_plan.cpp.
//
// Covers the paper's Section 2.2 transfer (pack / unpack around a chunk buffer) and the
// explicit device<->host copies of the CPU-forwarding variant (Section 2.1).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <mutex>
#include <new>
#include <optional>
#include <thread>
#include <vector>

#include "hxt_internal.h"
#include "hxt_kernels.h"

using namespace hxt;

// The plan: host tables, their device copies, and the checksum accumulators.
// Sender-side and receiver-side passes have separate sets (a pack on one stream and an unpack on another
// then never wait for each other); the _B sets serve the second of two message chains that run side by
// side on two streams (see chained_direct_stream).  SUM2 = the pair-of-sums passes: SEND for hxt_checksum2,
// hxt_seal and hxt_pack_seal, RECV for hxt_verify and hxt_unpack_verify.
enum Op {
    OP_PACK = 0, OP_UNPACK = 1, OP_CHECKSUM = 2, OP_SUM2_SEND = 3, OP_SUM2_RECV = 4,
    OP_PACK_B = 5, OP_UNPACK_B = 6, OP_SUM2_SEND_B = 7, OP_SUM2_RECV_B = 8, OP_COUNT = 9
};
inline bool op_keeps_pairs(int op) { return op == OP_SUM2_SEND || op == OP_SUM2_RECV || op == OP_SUM2_SEND_B || op == OP_SUM2_RECV_B; }

struct OpState {              // accumulator slots of one operation and who used them last
    uint8_t *acc = nullptr;
    bool used = false;
    hipStream_t last = nullptr;
    hipEvent_t ev = nullptr;
};

struct hxt_plan {
    Plan p;
    Tile *d_tiles = nullptr;
    uint32_t *d_chunk_tiles = nullptr;
    TensorDev *d_tensors = nullptr;
    uint32_t *d_inc = nullptr;                  // Plan::inc (tiles of the transpose that span chunks)
    uint32_t acc_stride = 0;
    uint32_t fan = 1;                           // first-level accumulator slots per chunk
    uint32_t sum_bits_table = 0, sum_bits_geom = 0;   // see slot_arrive: table-driven copies / closed-form kernels
    int device = -1;
    int nt_packed = -1;                         // HXT_OPT_PACKED_HINT: -1 by size, 0 cacheable, 1 non-temporal
    int stage_d2h_kernel = 0;                   // HXT_OPT_STAGE_D2H: 0 copy command, 1 the library's copy kernel
    OpState ops[OP_COUNT];
    std::recursive_mutex slots_mu;              // see SlotsLock
    // Events for hxt_exchange_stream, created on first need and kept until the plan is destroyed, so that a call
    // in steady state creates nothing.  A call borrows what it needs and hands it back when it has enqueued
    // everything (an event may be recorded again while earlier waits on it are still pending).
    std::mutex ev_mu;
    std::vector<hipEvent_t> ev_free;
};

// Accumulator slots for the entry point that may not allocate (hxt_pack_noalloc).  Every GPU the library
// runs on holds its own copy of this array until the process ends.  In host code the name is only a
// stand-in for the symbol: its device address is asked for once per device (scratch_on_device) and that
// pointer, never the name, is what kernels and fills receive.
constexpr size_t kScratchBytes = size_t(1) << 20;
constexpr uint32_t kScratchSlotStride = 256;
constexpr size_t kScratchSlots = kScratchBytes / kScratchSlotStride;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

// ---- host side --------------------------------------------------------------------

thread_local int g_last_hip = 0;

inline int hip_fail(hipError_t e)
{
    g_last_hip = int(e);
    return HXT_EHIP;
}

#define HXT_HIP(call)                                  \
    do {                                               \
        hipError_t e_ = (call);                        \
        if (e_ != hipSuccess) return hip_fail(e_);     \
    } while (0)

int env_int(const char *name, int dflt)
{
    const char *s = std::getenv(name);
    return (s && *s) ? std::atoi(s) : dflt;
}

// Cache hints.  Tensors are streamed once: non-temporal.  The packed buffer is written by
// pack and read back soon after (by the wire, or by unpack here): it stays cacheable while it
// can still be in the 256 MB last-level cache when it is re-read, and becomes non-temporal
// too for larger messages (measured: 56 MiB pack->unpack 21.1 us per kernel cacheable vs 22.7
// non-temporal; 1.7 GB 625 us vs 586 us).  HXT_NT_USER / HXT_NT_PACKED (0/1) override.
constexpr uint64_t kCacheablePackedLimit = uint64_t(128) << 20;

struct Tuning {
    int nt_user, nt_packed;        // -1 = automatic
    Tuning() : nt_user(env_int("HXT_NT_USER", -1)), nt_packed(env_int("HXT_NT_PACKED", -1)) {}
};
const Tuning &tuning()
{
    static Tuning t;
    return t;
}

inline bool packed_nontemporal(uint64_t packed_bytes)
{
    const int o = tuning().nt_packed;
    return o >= 0 ? o != 0 : packed_bytes > kCacheablePackedLimit;
}

inline bool packed_nontemporal(const hxt_plan_t &pl)
{
    return pl.nt_packed >= 0 ? pl.nt_packed != 0 : packed_nontemporal(pl.p.C * pl.p.B);
}

// Calls f.template operator()<NTU, NTP>() for the chosen cache hints.
template <typename F>
void with_hints(bool nt_packed, F &&f)
{
    const bool nt_user = tuning().nt_user != 0;
    if (nt_user) {
        if (nt_packed) f.template operator()<true, true>();
        else f.template operator()<true, false>();
    } else {
        if (nt_packed) f.template operator()<false, true>();
        else f.template operator()<false, false>();
    }
}

// The streaming copies are launched with 32 KiB of (unused) dynamic LDS per workgroup, which caps residency at 5
// workgroups per CU instead of 8: with 8 the memory system holds twice the bytes it needs to stay busy, every
// request queues for longer and the launch's tail grows.  Measured per launch, all-cold, checks on: k_uniform on
// 2 x 32 MiB 26.1 -> 25.3 us (23.9 -> 23.3 us with the packed side cacheable); k_contig on the 1.7 GB message 587 ->
// 557 us (6 per CU 574, 4 per CU 564, 3 per CU 563, 2 per CU 618); k_contig_tag 571 -> 559 us; k_contig_accumulate
// 717 -> 701 us.  Not applied where it does not pay: k_rows (23.1 -> 23.8 us), k_rows_split (30.7 -> 31.7 us),
// k_uniform_tag (27.3 vs 27.4 us all-cold, 25.5 vs 24.6 us cacheable), k_uniform_accumulate (no change).
// HXT_UNIFORM_LDS overrides (bytes, 0 = no cap).
constexpr int kUniformLdsPad = 32768;

inline size_t residency_cap_lds()
{
    static const size_t lds = size_t(std::max(0, std::min(65536, env_int("HXT_UNIFORM_LDS", kUniformLdsPad))));
    return lds;
}

template <int DIR, bool CSUM>
void launch_uniform(const UniformArgs &a, uint32_t tiles, bool nt_packed, hipStream_t st)
{
    const size_t lds = residency_cap_lds();
    with_hints(nt_packed, [&]<bool NTU, bool NTP>() { k_uniform<DIR, CSUM, NTU, NTP><<<tiles, kThreads, lds, st>>>(a); });
}

template <bool UNPACK, bool CSUM>
void launch_contig(const hxt_plan_t &pl, const Group &g, const BasePtrs &b, uint8_t *packed, const SumCtx &cx,
                   hipStream_t st)
{
    with_hints(packed_nontemporal(pl), [&]<bool NTU, bool NTP>() {
        k_contig<UNPACK, CSUM, NTU, NTP><<<g.count, kThreads, residency_cap_lds(), st>>>(pl.d_tiles + g.first, pl.d_chunk_tiles, b, packed, cx);
    });
}

template <bool UNPACK, bool CSUM>
void launch_rows(const hxt_plan_t &pl, const Group &g, const BasePtrs &b, uint8_t *packed, const SumCtx &cx,
                 hipStream_t st)
{
    with_hints(packed_nontemporal(pl), [&]<bool NTU, bool NTP>() {
        k_rows<UNPACK, CSUM, NTU, NTP><<<g.count, kThreads, 0, st>>>(pl.d_tiles + g.first, pl.d_chunk_tiles, pl.d_tensors,
                                                                     g.tensor_base, b, packed, cx);
    });
}

template <bool UNPACK, bool CSUM>
void launch_transpose(const hxt_plan_t &pl, uint32_t first, uint32_t count, int esize, const BasePtrs &b,
                      uint8_t *packed, const SumCtx &cx, hipStream_t st)
{
    const Tile *tiles = pl.d_tiles + first;
    const uint32_t *ct = pl.d_chunk_tiles;
    auto go = [&]<bool NTP>() {
        switch (esize) {
        case 1: k_transpose<uint8_t, UNPACK, CSUM, NTP><<<count, kThreads, 0, st>>>(tiles, ct, b, packed, cx); break;
        case 2: k_transpose<uint16_t, UNPACK, CSUM, NTP><<<count, kThreads, 0, st>>>(tiles, ct, b, packed, cx); break;
        case 4: k_transpose<uint32_t, UNPACK, CSUM, NTP><<<count, kThreads, 0, st>>>(tiles, ct, b, packed, cx); break;
        default: k_transpose<uint64_t, UNPACK, CSUM, NTP><<<count, kThreads, 0, st>>>(tiles, ct, b, packed, cx); break;
        }
    };
    if (packed_nontemporal(pl)) go.template operator()<true>();
    else go.template operator()<false>();
}

template <bool UNPACK, bool CSUM>
void launch_transpose_span(const hxt_plan_t &pl, uint32_t first, uint32_t count, int esize, const BasePtrs &b,
                           uint8_t *packed, const SumCtx &cx, hipStream_t st)
{
    const Tile *tiles = pl.d_tiles + first;
    const uint32_t *ct = pl.d_chunk_tiles, *inc = pl.d_inc;
    const ChunkGeom &g = pl.p.geom;
    auto go = [&]<bool NTP>() {
        switch (esize) {
        case 1: k_transpose_span<uint8_t, UNPACK, CSUM, NTP><<<count, kThreads, 0, st>>>(tiles, ct, inc, g, b, packed, cx); break;
        case 2: k_transpose_span<uint16_t, UNPACK, CSUM, NTP><<<count, kThreads, 0, st>>>(tiles, ct, inc, g, b, packed, cx); break;
        case 4: k_transpose_span<uint32_t, UNPACK, CSUM, NTP><<<count, kThreads, 0, st>>>(tiles, ct, inc, g, b, packed, cx); break;
        default: k_transpose_span<uint64_t, UNPACK, CSUM, NTP><<<count, kThreads, 0, st>>>(tiles, ct, inc, g, b, packed, cx); break;
        }
    };
    if (packed_nontemporal(pl)) go.template operator()<true>();
    else go.template operator()<false>();
}

template <bool UNPACK, bool CSUM>
void launch_generic(const hxt_plan_t &pl, uint32_t first, uint32_t count, uint32_t tensor_base, int esize,
                    const BasePtrs &b, uint8_t *packed, const SumCtx &cx, hipStream_t st)
{
    const Tile *tiles = pl.d_tiles + first;
    const uint32_t *ct = pl.d_chunk_tiles;
    const TensorDev *td = pl.d_tensors;
    auto go = [&]<bool NTP>() {
        switch (esize) {
        case 1: k_generic<uint8_t, UNPACK, CSUM, NTP><<<count, kThreads, 0, st>>>(tiles, ct, td, tensor_base, b, packed, cx); break;
        case 2: k_generic<uint16_t, UNPACK, CSUM, NTP><<<count, kThreads, 0, st>>>(tiles, ct, td, tensor_base, b, packed, cx); break;
        case 4: k_generic<uint32_t, UNPACK, CSUM, NTP><<<count, kThreads, 0, st>>>(tiles, ct, td, tensor_base, b, packed, cx); break;
        default: k_generic<uint64_t, UNPACK, CSUM, NTP><<<count, kThreads, 0, st>>>(tiles, ct, td, tensor_base, b, packed, cx); break;
        }
    };
    if (packed_nontemporal(pl)) go.template operator()<true>();
    else go.template operator()<false>();
}

// The accumulator slots of an operation are shared by all calls of that operation on this
// plan.  Calls on one stream are ordered by the stream; when the stream changes, the new
// stream is made to wait for everything enqueued so far on the previous one.  That only works
// if "enqueued so far" includes the previous claimant's kernels, so a call holds the plan's lock
// from its first claim until its launches are enqueued (host-side enqueue time only; one lock
// per plan, recursive because batched calls fall back to single calls).  Calls on different
// plans do not wait for each other.
using SlotsLock = std::lock_guard<std::recursive_mutex>;

// The locks of all the plans of a batched call, taken in address order (each plan once), so
// that two batched calls that share plans cannot wait for each other in a cycle.  Allocates
// nothing: every step looks for the lowest address above the one locked last.
class BatchLock {
  public:
    BatchLock(const hxt_plan_t *const *plans, int n) : plans_(plans), n_(n)
    {
        for (hxt_plan_t *pl = next(nullptr); pl; pl = next(pl)) pl->slots_mu.lock();
    }
    ~BatchLock()
    {
        for (hxt_plan_t *pl = next(nullptr); pl; pl = next(pl)) pl->slots_mu.unlock();
    }
    BatchLock(const BatchLock &) = delete;
    BatchLock &operator=(const BatchLock &) = delete;

  private:
    hxt_plan_t *next(const hxt_plan_t *after) const
    {
        const hxt_plan_t *best = nullptr;
        for (int i = 0; i < n_; ++i)
            if (plans_[i] && std::less<const hxt_plan_t *>()(after, plans_[i]) &&
                (!best || std::less<const hxt_plan_t *>()(plans_[i], best)))
                best = plans_[i];
        return const_cast<hxt_plan_t *>(best);
    }
    const hxt_plan_t *const *plans_;
    int n_;
};

int claim_slots(hxt_plan_t &pl, Op op, hipStream_t st, SumCtx &cx, uint64_t *sums)
{
    OpState &o = pl.ops[op];
    if (o.used && o.last != st) {
        if (!o.ev) HXT_HIP(hipEventCreateWithFlags(&o.ev, hipEventDisableTiming));
        if (hipEventRecord(o.ev, o.last) == hipSuccess)
            HXT_HIP(hipStreamWaitEvent(st, o.ev, 0));
        else
            (void)hipGetLastError();           // the previous stream no longer exists: nothing to wait for
    }
    o.used = true;
    o.last = st;
    cx.sums = sums;
    cx.acc = o.acc;
    cx.stride = pl.acc_stride;
    cx.sum_bits = 0;
    cx.fan = pl.fan;
    cx.chunks = uint32_t(pl.p.C);
    return HXT_OK;
}

// Bits a chunk's checksum can occupy (at most B/4 words below 2^32), if the arrival count of
// up to `arrivals` per slot still fits above them in a 64-bit word; else 0.
uint32_t single_word_bits(uint64_t chunk_bytes, uint32_t arrivals)
{
    uint32_t m = 0;
    while ((uint64_t(1) << m) < chunk_bytes / 4) ++m;
    uint32_t cb = 0;
    while ((uint64_t(1) << cb) <= arrivals) ++cb;
    return 32 + m + cb <= 64 ? 32 + m : 0;
}

// Most arrivals any slot sees when chunks of up to `tiles` tiles fan out over `fan` slots.
uint32_t max_arrivals(uint32_t tiles, uint32_t fan)
{
    return fan == 1 ? tiles : std::max((tiles + fan - 1) / fan, 2 * fan);
}

// First-level accumulator slots per chunk for chunks of up to `most` tiles: chunks of 128 tiles or more fan
// out over up to 16 slots so that a few dozen arrivals at most queue on one address (measured: a 25 MiB
// chunk of 1600 tiles loses 20 % without it, a 1 MiB chunk of 64 tiles is faster with a single slot).
uint32_t choose_fan(uint32_t most)
{
    uint32_t fan = 1;
    while (fan < 16 && most >= 128 * fan) fan *= 2;
    fan = uint32_t(std::max(1, std::min<int>(int(fan), env_int("HXT_FAN", 16))));
    while (fan & (fan - 1)) fan &= fan - 1;                               // keep a power of two
    return fan;
}

// Device address of this GPU's copy of `scratch`, looked up once per device with that device current.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
uint8_t *g_scratch_ptr[kMaxDevices] = {nullptr};

int scratch_on_device(uint8_t **out)
{
    int dev = -1;
    HXT_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return HXT_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        HXT_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return hip_fail(hipErrorInvalidSymbol);
        g_scratch_ptr[dev] = static_cast<uint8_t *>(ptr);
    }
    *out = g_scratch_ptr[dev];
    return HXT_OK;
}

template <bool UNPACK, bool CSUM>
int run_copy(hxt_plan_t &pl, void *const *ptrs, uint8_t *packed, uint64_t *sums, hipStream_t st, int chain = 0)
{
    const Plan &p = pl.p;
    SumCtx cx{nullptr, nullptr, 0, 0, 1, 0};
    std::optional<SlotsLock> lock;
    if constexpr (CSUM) {
        lock.emplace(pl.slots_mu);
        const Op op = chain ? (UNPACK ? OP_UNPACK_B : OP_PACK_B) : (UNPACK ? OP_UNPACK : OP_PACK);
        int rc = claim_slots(pl, op, st, cx, sums);
        if (rc != HXT_OK) return rc;
        cx.sum_bits = pl.sum_bits_table;
    }
    if (p.uniform) {
        uint8_t *base = static_cast<uint8_t *>(ptrs[p.uniform_tensor]);
        cx.sum_bits = pl.sum_bits_geom;
        UniformArgs a;
        std::memset(&a, 0, sizeof a);
        a.n = 1;
        a.it[0] = UniformItem{p.geom, base, packed, cx, 0, UNPACK};
        if (reinterpret_cast<uintptr_t>(base) % 16 == 0)
            launch_uniform<UNPACK ? DIR_UNPACK : DIR_PACK, CSUM>(a, p.geom.ntiles, packed_nontemporal(pl), st);
        else                                             // element aligned only: narrower accesses on the tensor side
            k_uniform_any<UNPACK, CSUM><<<p.geom.ntiles, kThreads, 0, st>>>(a);
        HXT_HIP(hipGetLastError());
        return HXT_OK;
    }
    for (const Group &g : p.groups) {
        BasePtrs b;
        std::memset(&b, 0, sizeof b);
        bool fast_ok = true;
        for (uint32_t i = 0; i < g.n_tensors; ++i) {
            const TensorPlan &tp = p.tensors[g.tensor_base + i];
            uint8_t *base = static_cast<uint8_t *>(ptrs[g.tensor_base + i]);
            b.p[i] = base;
            if (tp.bytes && tp.kind == g.kernel && reinterpret_cast<uintptr_t>(base) % 16) fast_ok = false;
        }
        if (g.kernel == K_CONTIG && fast_ok) {
            launch_contig<UNPACK, CSUM>(pl, g, b, packed, cx, st);
        } else if (g.kernel == K_CONTIG) {               // some base is element aligned only
            k_contig_any<UNPACK, CSUM><<<g.count, kThreads, 0, st>>>(pl.d_tiles + g.first, pl.d_chunk_tiles, b, packed, cx);
        } else if (g.kernel == K_ROWS && fast_ok) {
            launch_rows<UNPACK, CSUM>(pl, g, b, packed, cx, st);
        } else if (g.kernel == K_ROWS) {
            k_rows_any<UNPACK, CSUM><<<g.count, kThreads, 0, st>>>(pl.d_tiles + g.first, pl.d_chunk_tiles, pl.d_tensors,
                                                                   g.tensor_base, b, packed, cx);
        } else if (g.kernel == K_ROWS_SPLIT) {
            if (packed_nontemporal(pl))
                k_rows_split<UNPACK, CSUM, true><<<g.count, kThreads, 0, st>>>(pl.d_tiles + g.first, pl.d_chunk_tiles, pl.d_tensors,
                                                                               g.tensor_base, b, packed, cx);
            else
                k_rows_split<UNPACK, CSUM, false><<<g.count, kThreads, 0, st>>>(pl.d_tiles + g.first, pl.d_chunk_tiles, pl.d_tensors,
                                                                                g.tensor_base, b, packed, cx);
        } else {
            // The transpose and per-element kernels are instantiated per element size: issue one
            // launch per run of tiles whose tensors share it (host table, same order as on the device).
            uint32_t i = 0;
            while (i < g.count) {
                const int es = p.tensors[g.tensor_base + p.tiles[g.first + i].tensor].esize;
                uint32_t j = i + 1;
                while (j < g.count && p.tensors[g.tensor_base + p.tiles[g.first + j].tensor].esize == es) ++j;
                if (g.kernel == K_TRANSPOSE)
                    launch_transpose<UNPACK, CSUM>(pl, g.first + i, j - i, es, b, packed, cx, st);
                else if (g.kernel == K_TRANSPOSE_SPAN)
                    launch_transpose_span<UNPACK, CSUM>(pl, g.first + i, j - i, es, b, packed, cx, st);
                else
                    launch_generic<UNPACK, CSUM>(pl, g.first + i, j - i, g.tensor_base, es, b, packed, cx, st);
                i = j;
            }
        }
        HXT_HIP(hipGetLastError());
    }
    return HXT_OK;
}

// Receive and accumulate: contiguous bf16 / f32 tensors with 16-byte aligned bases only.
template <bool CSUM>
int run_accumulate(hxt_plan_t &pl, void *const *ptrs, uint8_t *packed, uint64_t *sums, hipStream_t st)
{
    const Plan &p = pl.p;
    SumCtx cx{nullptr, nullptr, 0, 0, 1, 0};
    std::optional<SlotsLock> lock;
    if constexpr (CSUM) {
        lock.emplace(pl.slots_mu);
        int rc = claim_slots(pl, OP_UNPACK, st, cx, sums);
        if (rc != HXT_OK) return rc;
        cx.sum_bits = pl.sum_bits_table;
    }
    const bool ntp = packed_nontemporal(pl);
    if (p.uniform) {
        const TensorPlan &tp = p.tensors[p.uniform_tensor];
        UniformArgs a;
        std::memset(&a, 0, sizeof a);
        a.n = 1;
        cx.sum_bits = CSUM ? pl.sum_bits_geom : 0;
        // `unpack` carries the element kind here: 1 = f32, 0 = bf16
        a.it[0] = UniformItem{p.geom, static_cast<uint8_t *>(ptrs[p.uniform_tensor]), packed, cx, 0,
                              tp.dtype == HXT_F32 ? 1u : 0u};
        if (reinterpret_cast<uintptr_t>(ptrs[p.uniform_tensor]) % 16 == 0)
            with_hints(ntp, [&]<bool NTU, bool NTP>() {
                k_uniform_accumulate<CSUM, NTU, NTP><<<p.geom.ntiles, kThreads, 0, st>>>(a);
            });
        else
            k_uniform_accumulate_any<CSUM><<<p.geom.ntiles, kThreads, 0, st>>>(a);
        HXT_HIP(hipGetLastError());
        return HXT_OK;
    }
    for (const Group &g : p.groups) {                      // only K_CONTIG groups exist in such a plan
        BasePtrs b;
        ElemKinds kinds;
        std::memset(&b, 0, sizeof b);
        std::memset(&kinds, 0, sizeof kinds);
        bool aligned = true;
        for (uint32_t i = 0; i < g.n_tensors; ++i) {
            b.p[i] = static_cast<uint8_t *>(ptrs[g.tensor_base + i]);
            kinds.f32[i] = p.tensors[g.tensor_base + i].dtype == HXT_F32;
            if (p.tensors[g.tensor_base + i].bytes && reinterpret_cast<uintptr_t>(b.p[i]) % 16) aligned = false;
        }
        if (aligned)
            with_hints(ntp, [&]<bool NTU, bool NTP>() {
                k_contig_accumulate<CSUM, NTU, NTP><<<g.count, kThreads, residency_cap_lds(), st>>>(pl.d_tiles + g.first, pl.d_chunk_tiles,
                                                                                  b, kinds, packed, cx);
            });
        else
            k_contig_accumulate_any<CSUM><<<g.count, kThreads, 0, st>>>(pl.d_tiles + g.first, pl.d_chunk_tiles, b, kinds,
                                                                        packed, cx);
        HXT_HIP(hipGetLastError());
    }
    return HXT_OK;
}

int check_common(const hxt_plan_t *plan, const void *packed)
{
    if (!plan) return HXT_EINVAL;
    const Plan &p = plan->p;
    if (p.C == 0) return HXT_OK;
    if (!packed) return HXT_EINVAL;
    if (reinterpret_cast<uintptr_t>(packed) % HXT_ALIGN) return HXT_EALIGN;
    if (plan->device < 0 || !plan->ops[0].acc) {
        g_last_hip = int(hipErrorNoDevice);
        return HXT_EHIP;
    }
    int cur = -1;
    if (hipGetDevice(&cur) != hipSuccess || cur != plan->device) {     // the work tables live on the plan's device
        (void)hipGetLastError();
        g_last_hip = int(hipErrorInvalidDevice);
        return HXT_EHIP;
    }
    return HXT_OK;
}

int check_tensor_pointers(const Plan &p, void *const *ptrs)
{
    if (!ptrs) return HXT_EINVAL;
    for (size_t i = 0; i < p.tensors.size(); ++i) {
        if (p.tensors[i].bytes == 0) continue;
        if (!ptrs[i]) return HXT_EINVAL;
        if (reinterpret_cast<uintptr_t>(ptrs[i]) % p.tensors[i].esize) return HXT_EALIGN;
    }
    return HXT_OK;
}

template <typename T>
int to_device(T **dst, const std::vector<T> &src)
{
    if (src.empty()) return HXT_OK;
    HXT_HIP(hipMalloc(reinterpret_cast<void **>(dst), src.size() * sizeof(T)));
    HXT_HIP(hipMemcpy(*dst, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice));
    return HXT_OK;
}

int upload(hxt_plan_t &pl)
{
    pl.nt_packed = tuning().nt_packed;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return HXT_OK;                      // no GPU: queries still work, data-plane calls report HXT_EHIP
    }
    pl.device = dev;
    const Plan &p = pl.p;
    if (p.C == 0) return HXT_OK;
    int rc;
    if ((rc = to_device(&pl.d_tiles, p.tiles)) != HXT_OK) return rc;
    if ((rc = to_device(&pl.d_chunk_tiles, p.chunk_tiles)) != HXT_OK) return rc;
    if ((rc = to_device(&pl.d_tensors, p.tdev)) != HXT_OK) return rc;
    if (!p.inc.empty() && (rc = to_device(&pl.d_inc, p.inc)) != HXT_OK) return rc;
    // Accumulator slots: fan-out as choose_fan says; slots are 256 bytes apart (separate memory
    // channels) unless that would be large.
    uint32_t most = p.geom.tpc;
    for (uint32_t n : p.chunk_tiles) most = std::max(most, n);
    pl.fan = choose_fan(most);
    const bool two_word = env_int("HXT_TWO_WORD_COMMIT", 0) != 0;
    uint32_t most_table = 0;
    for (uint32_t n : p.chunk_tiles) most_table = std::max(most_table, n);
    pl.sum_bits_table = two_word ? 0 : single_word_bits(p.B, max_arrivals(most_table, pl.fan));
    pl.sum_bits_geom = two_word ? 0 : single_word_bits(p.B, max_arrivals(p.geom.tpc, pl.fan));
    const size_t slots = size_t(p.C) * (pl.fan + 1);
    pl.acc_stride = slots <= 65536 ? 256 : uint32_t(sizeof(Acc));
    const size_t bytes = slots * pl.acc_stride;
    for (int i = 0; i < OP_COUNT; ++i) {
        const size_t n = op_keeps_pairs(i) ? 2 * bytes + 2 * pl.acc_stride : bytes;   // pairs of slots, plus one pair that counts finished chunks
        HXT_HIP(hipMalloc(reinterpret_cast<void **>(&pl.ops[i].acc), n));
        HXT_HIP(hipMemset(pl.ops[i].acc, 0, n));
    }
    HXT_HIP(hipDeviceSynchronize());
    return HXT_OK;
}

// Byte ranges of the packed buffer that staging moves for a lane selection.
int stage_ranges(const Plan &p, int lane, uint64_t (*r)[2])
{
    auto used = [&](int l) -> uint64_t {
        uint64_t n = p.lane_chunks[l];
        if (n == 0) return 0;
        return (n - 1) * p.B + p.chunk_padded((n - 1) * p.k + l);
    };
    if (lane >= 0) {
        r[0][0] = p.lane_off[lane];
        r[0][1] = used(lane);
        return r[0][1] ? 1 : 0;
    }
    // all lanes: regions are adjacent; only the lane holding the last chunk can end short
    if (p.C == 0) return 0;
    const int ls = int((p.C - 1) % p.k);
    const uint64_t cut = p.lane_off[ls] + used(ls), total = p.lane_off[p.k];
    r[0][0] = 0;
    if (cut == p.lane_off[ls + 1]) {
        r[0][1] = total;
        return 1;
    }
    r[0][1] = cut;
    if (p.lane_off[ls + 1] == total) return 1;
    r[1][0] = p.lane_off[ls + 1];
    r[1][1] = total - p.lane_off[ls + 1];
    return 2;
}

// Workgroups of the staging copy kernel: enough to keep the host link busy (it needs about 100 KB in flight;
// measured 55 GB/s with 16 workgroups and with 4096), few enough to leave the chip to the kernels beside it.
constexpr uint32_t kStageCopyGroups = 64;

int copy_range(const void *from, void *to, uint64_t off, uint64_t bytes, hipMemcpyKind kind, bool by_kernel, hipStream_t st)
{
    const uint8_t *f = static_cast<const uint8_t *>(from) + off;
    uint8_t *t = static_cast<uint8_t *>(to) + off;
    if (by_kernel) {                                   // offsets and lengths are multiples of 256
        static const uint32_t groups = uint32_t(std::max(1, std::min(4096, env_int("HXT_STAGE_GROUPS", int(kStageCopyGroups)))));
        k_stage_copy<<<groups, kThreads, 0, st>>>(reinterpret_cast<u32x4 *>(t), reinterpret_cast<const u32x4 *>(f), bytes / 16);
        HXT_HIP(hipGetLastError());
        return HXT_OK;
    }
    HXT_HIP(hipMemcpyAsync(t, f, bytes, kind, st));
    return HXT_OK;
}

int stage(const hxt_plan_t *plan, int lane, int64_t first_slot, int64_t n_slots, const void *from, void *to, hipMemcpyKind kind,
          void *stream)
{
    if (!plan) return HXT_EINVAL;
    const Plan &p = plan->p;
    if (lane < -1 || lane >= p.k) return HXT_EINVAL;
    if (n_slots >= 0 && (lane < 0 || first_slot < 0 || uint64_t(first_slot) + uint64_t(n_slots) > p.lane_chunks[lane])) return HXT_EINVAL;
    if (p.C == 0 || n_slots == 0) return HXT_OK;
    if (!from || !to) return HXT_EINVAL;
    if (reinterpret_cast<uintptr_t>(from) % HXT_ALIGN || reinterpret_cast<uintptr_t>(to) % HXT_ALIGN) return HXT_EALIGN;
    const bool by_kernel = kind == hipMemcpyDeviceToHost && plan->stage_d2h_kernel > 0;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (n_slots > 0) {                                 // a run of slots of one lane: full slots, the lane's last one up to its padded end
        const uint64_t last = uint64_t(first_slot + n_slots - 1) * p.k + lane;       // the chunk in the run's last slot
        const uint64_t bytes = uint64_t(n_slots - 1) * p.B + p.chunk_padded(last);
        return copy_range(from, to, p.lane_off[lane] + uint64_t(first_slot) * p.B, bytes, kind, by_kernel, st);
    }
    uint64_t r[2][2];
    const int n = stage_ranges(p, lane, r);
    for (int i = 0; i < n; ++i) {
        int rc = copy_range(from, to, r[i][0], r[i][1], kind, by_kernel, st);
        if (rc != HXT_OK) return rc;
    }
    return HXT_OK;
}

// Batch: the messages that the uniform kernel can take (one contiguous 16-byte aligned tensor,
// same checksum choice) are fused, up to kMaxBatch per launch; the rest go one by one.
template <bool UNPACK>
int run_batch(int n, const hxt_plan_t *const *plans, void *const *const *tensors, void *const *packed,
              uint64_t *const *sums, hipStream_t st)
{
    if (n < 0 || (n > 0 && (!plans || !tensors || !packed))) return HXT_EINVAL;
    for (int i = 0; i < n; ++i) {                      // validate everything before enqueuing anything
        int rc = check_common(plans[i], packed[i]);
        if (rc != HXT_OK) return rc;
        if (plans[i]->p.C == 0) continue;
        if ((rc = check_tensor_pointers(plans[i]->p, tensors[i])) != HXT_OK) return rc;
        if (UNPACK && !plans[i]->p.all_unpack_safe) return HXT_EOVERLAP;
        for (int j = 0; j < i; ++j)
            if (plans[j] == plans[i] && sums && sums[i] && sums[j]) return HXT_EINVAL;   // one accumulator set per plan
    }
    BatchLock lock(plans, n);
    int i = 0;
    while (i < n) {
        hxt_plan_t &pl = *const_cast<hxt_plan_t *>(plans[i]);
        const Plan &p = pl.p;
        uint64_t *sm = sums ? sums[i] : nullptr;
        auto fusable = [&](int j) {
            const Plan &q = plans[j]->p;
            return q.C != 0 && q.uniform && reinterpret_cast<uintptr_t>(tensors[j][q.uniform_tensor]) % 16 == 0 &&
                   ((sums ? sums[j] : nullptr) != nullptr) == (sm != nullptr);
        };
        if (p.C == 0) {
            ++i;
            continue;
        }
        if (!fusable(i)) {
            uint8_t *pk = static_cast<uint8_t *>(packed[i]);
            int rc = sm ? run_copy<UNPACK, true>(pl, tensors[i], pk, sm, st) : run_copy<UNPACK, false>(pl, tensors[i], pk, nullptr, st);
            if (rc != HXT_OK) return rc;
            ++i;
            continue;
        }
        UniformArgs a;
        std::memset(&a, 0, sizeof a);
        uint64_t tiles = 0, bytes = 0;
        int j = i;
        while (j < n && a.n < uint32_t(kMaxBatch) && fusable(j) && tiles + plans[j]->p.geom.ntiles < (uint64_t(1) << 31)) {
            hxt_plan_t &pj = *const_cast<hxt_plan_t *>(plans[j]);
            SumCtx cx{nullptr, nullptr, 0, 0, 1, 0};
            if (sm) {
                int rc = claim_slots(pj, UNPACK ? OP_UNPACK : OP_PACK, st, cx, sums[j]);
                if (rc != HXT_OK) return rc;
                cx.sum_bits = pj.sum_bits_geom;
            }
            a.it[a.n++] = UniformItem{pj.p.geom, static_cast<uint8_t *>(tensors[j][pj.p.uniform_tensor]),
                                      static_cast<uint8_t *>(packed[j]), cx, uint32_t(tiles), UNPACK};
            tiles += pj.p.geom.ntiles;
            bytes += pj.p.C * pj.p.B;
            ++j;
        }
        constexpr int DIR = UNPACK ? DIR_UNPACK : DIR_PACK;
        // cache hint of the launch: the first message's plan decides if it has been told to, else the bytes of the launch
        const bool ntp = plans[i]->nt_packed >= 0 ? plans[i]->nt_packed != 0 : packed_nontemporal(bytes);
        if (sm) launch_uniform<DIR, true>(a, uint32_t(tiles), ntp, st);
        else launch_uniform<DIR, false>(a, uint32_t(tiles), ntp, st);
        HXT_HIP(hipGetLastError());
        i = j;
    }
    return HXT_OK;
}

// The three users of the pair-of-sums pass.
int run_sum2(const hxt_plan_t *plan, const void *packed, int mode, void *out, const TagWork &work, void *stream,
             int chain = 0)
{
    int rc = check_common(plan, packed);
    if (rc != HXT_OK) return rc;
    if (!out || (mode == SUM2_VERIFY && !work.tags)) return HXT_EINVAL;
    const uintptr_t align = mode == SUM2_SEAL ? 16 : (mode == SUM2_VERIFY ? 4 : 8);
    if (reinterpret_cast<uintptr_t>(out) % align) return HXT_EALIGN;
    if (mode == SUM2_VERIFY && reinterpret_cast<uintptr_t>(work.tags) % 16) return HXT_EALIGN;
    hxt_plan_t &pl = *const_cast<hxt_plan_t *>(plan);
    hipStream_t st = static_cast<hipStream_t>(stream);
    SumCtx cx{nullptr, nullptr, 0, 0, 1, 0};          // callers have dealt with the empty message
    SlotsLock lock(pl.slots_mu);
    if ((rc = claim_slots(pl, mode == SUM2_VERIFY ? (chain ? OP_SUM2_RECV_B : OP_SUM2_RECV) : (chain ? OP_SUM2_SEND_B : OP_SUM2_SEND), st, cx, nullptr)) != HXT_OK) return rc;
    const uint8_t *pk = static_cast<const uint8_t *>(packed);
    const bool ntp = packed_nontemporal(pl);
    auto launch = [&]<int MODE>() {
        TagWork w = work;
        w.sum_bits = pl.sum_bits_geom;
        if (ntp) k_checksum2<MODE, true><<<pl.p.geom.ntiles, kThreads, 0, st>>>(pl.p.geom, pk, out, cx.acc, cx.stride, cx.fan, w);
        else k_checksum2<MODE, false><<<pl.p.geom.ntiles, kThreads, 0, st>>>(pl.p.geom, pk, out, cx.acc, cx.stride, cx.fan, w);
    };
    if (mode == SUM2_SUMS) launch.template operator()<SUM2_SUMS>();
    else if (mode == SUM2_SEAL) launch.template operator()<SUM2_SEAL>();
    else launch.template operator()<SUM2_VERIFY>();
    HXT_HIP(hipGetLastError());
    return HXT_OK;
}

// pack + seal (UNPACK = false) or unpack + verify (UNPACK = true).  One pass for a message that is one
// contiguous, 16-byte aligned tensor; otherwise the copy and the pair-of-sums pass one after the other
// on the stream, which gives the same bytes, tags and masks.
template <bool UNPACK>
int run_copy_tag(const hxt_plan_t *plan, void *const *ptrs, void *packed, void *out, const TagWork &work, void *stream,
                 int chain = 0)
{
    constexpr int MODE = UNPACK ? SUM2_VERIFY : SUM2_SEAL;
    int rc = check_common(plan, packed);
    if (rc != HXT_OK) return rc;
    if ((rc = check_tensor_pointers(plan->p, ptrs)) != HXT_OK) return rc;
    if (!out || (UNPACK && !work.tags)) return HXT_EINVAL;
    if (reinterpret_cast<uintptr_t>(out) % (UNPACK ? 4 : 16)) return HXT_EALIGN;
    if (UNPACK && reinterpret_cast<uintptr_t>(work.tags) % 16) return HXT_EALIGN;
    if (UNPACK && !plan->p.all_unpack_safe) return HXT_EOVERLAP;
    hxt_plan_t &pl = *const_cast<hxt_plan_t *>(plan);
    const Plan &p = pl.p;
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint8_t *pk = static_cast<uint8_t *>(packed);
    uint8_t *base = p.uniform ? static_cast<uint8_t *>(ptrs[p.uniform_tensor]) : nullptr;
    bool aligned = true;                                 // every live tensor's base on a 16-byte boundary
    for (size_t i = 0; i < p.tensors.size(); ++i)
        aligned = aligned && (p.tensors[i].bytes == 0 || reinterpret_cast<uintptr_t>(ptrs[i]) % 16 == 0);
    const bool one_pass = aligned && (p.uniform || p.all_contig);
    if (!one_pass) {
        if (UNPACK) {                                    // check what arrived, then scatter it
            if ((rc = run_sum2(plan, packed, MODE, out, work, stream, chain)) != HXT_OK) return rc;
            return run_copy<true, false>(pl, ptrs, pk, nullptr, st, chain);
        }
        if ((rc = run_copy<false, false>(pl, ptrs, pk, nullptr, st, chain)) != HXT_OK) return rc;
        return run_sum2(plan, packed, MODE, out, work, stream, chain);
    }
    SumCtx cx{nullptr, nullptr, 0, 0, 1, 0};
    SlotsLock lock(pl.slots_mu);
    if ((rc = claim_slots(pl, UNPACK ? (chain ? OP_SUM2_RECV_B : OP_SUM2_RECV) : (chain ? OP_SUM2_SEND_B : OP_SUM2_SEND), st, cx, nullptr)) != HXT_OK) return rc;
    TagWork w = work;
    if (p.uniform) {
        w.sum_bits = pl.sum_bits_geom;
        UniformTagArgs a;
        std::memset(&a, 0, sizeof a);
        a.n = 1;
        a.it[0] = UniformTagItem{p.geom, base, pk, out, cx.acc, cx.stride, cx.fan, w, 0};
        with_hints(packed_nontemporal(pl), [&]<bool NTU, bool NTP>() {
            k_uniform_tag<UNPACK, MODE, NTU, NTP><<<p.geom.ntiles, kThreads, 0, st>>>(a);
        });
        HXT_HIP(hipGetLastError());
        return HXT_OK;
    }
    // contiguous tensors of a multi-tensor message: the table-driven copy with both sums taken on the way; the
    // chunks' accumulators carry over from one launch group to the next
    w.sum_bits = pl.sum_bits_table;
    for (const Group &g : p.groups) {
        BasePtrs b;
        std::memset(&b, 0, sizeof b);
        for (uint32_t i = 0; i < g.n_tensors; ++i) b.p[i] = static_cast<uint8_t *>(ptrs[g.tensor_base + i]);
        with_hints(packed_nontemporal(pl), [&]<bool NTU, bool NTP>() {
            k_contig_tag<UNPACK, MODE, NTU, NTP><<<g.count, kThreads, residency_cap_lds(), st>>>(pl.d_tiles + g.first, pl.d_chunk_tiles, b, pk,
                                                                               p.geom, out, cx.acc, cx.stride, cx.fan, w);
        });
        HXT_HIP(hipGetLastError());
    }
    return HXT_OK;
}

// Batched pack + seal / unpack + verify: messages that are one contiguous 16-byte aligned tensor share
// launches (up to kMaxBatch each), the rest go one by one.
template <bool UNPACK>
int run_tag_batch(int n, const hxt_plan_t *const *plans, void *const *const *tensors, void *const *packed,
                  void *const *outs, const hxt_chunk_tag_t *const *tags_in, const uint64_t *seq,
                  const uint32_t *micro_batch, hipStream_t st)
{
    constexpr int MODE = UNPACK ? SUM2_VERIFY : SUM2_SEAL;
    if (n < 0 || (n > 0 && (!plans || !tensors || !packed || !outs || !seq || !micro_batch || (UNPACK && !tags_in))))
        return HXT_EINVAL;
    for (int i = 0; i < n; ++i) {                      // validate everything before enqueuing anything
        if (!plans[i]) return HXT_EINVAL;
        if (plans[i]->p.C == 0) {
            if (UNPACK && !outs[i]) return HXT_EINVAL;
            continue;
        }
        int rc = check_common(plans[i], packed[i]);
        if (rc != HXT_OK) return rc;
        if ((rc = check_tensor_pointers(plans[i]->p, tensors[i])) != HXT_OK) return rc;
        if (!outs[i] || (UNPACK && !tags_in[i])) return HXT_EINVAL;
        if (reinterpret_cast<uintptr_t>(outs[i]) % (UNPACK ? 4 : 16)) return HXT_EALIGN;
        if (UNPACK && reinterpret_cast<uintptr_t>(tags_in[i]) % 16) return HXT_EALIGN;
        if (UNPACK && !plans[i]->p.all_unpack_safe) return HXT_EOVERLAP;
        for (int j = 0; j < i; ++j)
            if (plans[j] == plans[i]) return HXT_EINVAL;     // one accumulator set per plan
    }
    BatchLock lock(plans, n);
    int i = 0;
    while (i < n) {
        auto work_of = [&](int j) {
            return TagWork{UNPACK ? reinterpret_cast<const uint8_t *>(tags_in[j]) : nullptr, seq[j], micro_batch[j], 0};
        };
        auto fusable = [&](int j) {
            const Plan &q = plans[j]->p;
            return q.C != 0 && q.uniform && reinterpret_cast<uintptr_t>(tensors[j][q.uniform_tensor]) % 16 == 0;
        };
        if (!fusable(i)) {
            int rc;
            if (plans[i]->p.C == 0)
                rc = UNPACK ? hxt_verify(plans[i], packed[i], tags_in[i], seq[i], micro_batch[i], static_cast<uint32_t *>(outs[i]), st)
                            : HXT_OK;
            else
                rc = run_copy_tag<UNPACK>(plans[i], tensors[i], packed[i], outs[i], work_of(i), st);
            if (rc != HXT_OK) return rc;
            ++i;
            continue;
        }
        UniformTagArgs a;
        std::memset(&a, 0, sizeof a);
        uint64_t tiles = 0, bytes = 0;
        int j = i;
        while (j < n && a.n < uint32_t(kMaxBatch) && fusable(j) && tiles + plans[j]->p.geom.ntiles < (uint64_t(1) << 31)) {
            hxt_plan_t &pj = *const_cast<hxt_plan_t *>(plans[j]);
            SumCtx cx{nullptr, nullptr, 0, 0, 1, 0};
            int rc = claim_slots(pj, UNPACK ? OP_SUM2_RECV : OP_SUM2_SEND, st, cx, nullptr);
            if (rc != HXT_OK) return rc;
            TagWork w = work_of(j);
            w.sum_bits = pj.sum_bits_geom;
            a.it[a.n++] = UniformTagItem{pj.p.geom, static_cast<uint8_t *>(tensors[j][pj.p.uniform_tensor]),
                                         static_cast<uint8_t *>(packed[j]), outs[j], cx.acc, cx.stride, cx.fan, w, uint32_t(tiles)};
            tiles += pj.p.geom.ntiles;
            bytes += pj.p.C * pj.p.B;
            ++j;
        }
        const bool ntp = plans[i]->nt_packed >= 0 ? plans[i]->nt_packed != 0 : packed_nontemporal(bytes);
        with_hints(ntp, [&]<bool NTU, bool NTP>() { k_uniform_tag<UNPACK, MODE, NTU, NTP><<<uint32_t(tiles), kThreads, 0, st>>>(a); });
        HXT_HIP(hipGetLastError());
        i = j;
    }
    return HXT_OK;
}

// n events from the plan's pool (created if the pool runs short); false after a HIP error (out is then empty).
bool borrow_events(hxt_plan_t &pl, size_t n, std::vector<hipEvent_t> &out)
{
    std::lock_guard<std::mutex> lock(pl.ev_mu);
    out.clear();
    try {                                              // room for every event on both sides: nothing below can throw
        out.reserve(n);
        pl.ev_free.reserve(pl.ev_free.size() + n);
    } catch (const std::bad_alloc &) {
        g_last_hip = int(hipErrorOutOfMemory);
        return false;
    }
    while (out.size() < n) {
        hipEvent_t e = nullptr;
        if (!pl.ev_free.empty()) {
            e = pl.ev_free.back();
            pl.ev_free.pop_back();
        } else if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) {
            g_last_hip = int(hipGetLastError());
            for (hipEvent_t b : out) pl.ev_free.push_back(b);
            out.clear();
            return false;
        }
        out.push_back(e);
    }
    return true;
}

void return_events(hxt_plan_t &pl, std::vector<hipEvent_t> &ev)
{
    std::lock_guard<std::mutex> lock(pl.ev_mu);
    for (hipEvent_t e : ev) pl.ev_free.push_back(e);
    ev.clear();
}

// Device-direct micro-batch stream for single-tensor messages, without cross-stream handshakes:
// launch k unpacks message k-1 and packs message k (different buffer sets, independent work, so
// the two overlap inside the launch and fill each other's ramp-up and tail); consecutive launches
// on one stream carry the pack -> unpack dependency.  The other two streams are made to wait for
// the last launch, so that draining any of the three means every message has arrived.
int fused_direct_stream(hxt_plan_t &pl, const hxt_exchange_t &x, hipStream_t sp, hipStream_t ss, hipStream_t su)
{
    const Plan &p = pl.p;
    const size_t T = p.tensors.size();
    const bool nt_packed = packed_nontemporal(pl);
    SlotsLock lock(pl.slots_mu);
    for (int k = 0; k <= x.n_messages; ++k) {
        UniformArgs a;
        std::memset(&a, 0, sizeof a);
        uint32_t tiles = 0;
        auto add = [&](int msg, bool unpack) -> int {
            SumCtx cx{nullptr, nullptr, 0, 0, 1, 0};
            uint64_t *sm = unpack ? x.recv_sums : x.send_sums;
            if (sm) {
                int rc = claim_slots(pl, unpack ? OP_UNPACK : OP_PACK, sp, cx, sm + size_t(msg) * p.C);
                if (rc != HXT_OK) return rc;
                cx.sum_bits = pl.sum_bits_geom;
            }
            void *user = unpack ? x.dst[msg * T + p.uniform_tensor] : const_cast<void *>(x.src[msg * T + p.uniform_tensor]);
            a.it[a.n++] = UniformItem{p.geom, static_cast<uint8_t *>(user),
                                      static_cast<uint8_t *>(x.packed_send[msg % x.n_buffers]), cx, tiles, unpack ? 1u : 0u};
            tiles += p.geom.ntiles;
            return HXT_OK;
        };
        int rc = HXT_OK;
        if (k > 0) rc = add(k - 1, true);
        if (rc == HXT_OK && k < x.n_messages) rc = add(k, false);
        if (rc != HXT_OK) return rc;
        if (x.send_sums) launch_uniform<DIR_MIXED, true>(a, tiles, nt_packed, sp);
        else launch_uniform<DIR_MIXED, false>(a, tiles, nt_packed, sp);
        HXT_HIP(hipGetLastError());
    }
    if (su != sp || ss != sp) {
        std::vector<hipEvent_t> done;
        if (!borrow_events(pl, 1, done)) return HXT_EHIP;
        hipError_t e = hipEventRecord(done[0], sp);
        if (e == hipSuccess && su != sp) e = hipStreamWaitEvent(su, done[0], 0);
        if (e == hipSuccess && ss != sp) e = hipStreamWaitEvent(ss, done[0], 0);
        return_events(pl, done);
        if (e != hipSuccess) return hip_fail(e);
    }
    return HXT_OK;
}

// Device-direct micro-batch stream as two chains: even messages on stream a, odd messages on stream
// b, each chain packing and unpacking its own messages in stream order.  With an even number of
// buffer sets a buffer only ever serves one chain, so the chains share nothing (each has its own
// accumulator slots) and need no events; their kernels overlap and fill each other's ramp-up and
// tail.  The third stream is made to wait for both, so that draining any of the three means every
// message has arrived.
int chained_direct_stream(hxt_plan_t &pl, const hxt_exchange_t &x, hipStream_t a, hipStream_t b, hipStream_t third)
{
    const Plan &p = pl.p;
    const size_t T = p.tensors.size();
    for (int i = 0; i < x.n_messages; ++i) {
        const int chain = i & 1;
        hipStream_t st = chain ? b : a;
        uint8_t *buf = static_cast<uint8_t *>(x.packed_send[i % x.n_buffers]);
        void *const *src = const_cast<void *const *>(x.src + i * T);
        uint64_t *s_send = x.send_sums ? x.send_sums + size_t(i) * p.C : nullptr;
        uint64_t *s_recv = x.recv_sums ? x.recv_sums + size_t(i) * p.C : nullptr;
        int rc;
        if (x.tags_send) {                               // sealed and verified inside the copies
            void *tags = x.tags_send[i % x.n_buffers];
            const uint64_t seq = x.seq_base + uint64_t(i);
            rc = run_copy_tag<false>(&pl, src, buf, tags, TagWork{nullptr, seq, uint32_t(i), 0}, st, chain);
            if (rc != HXT_OK) return rc;
            rc = run_copy_tag<true>(&pl, x.dst + i * T, buf, x.status + size_t(i) * (p.C + 1),
                                    TagWork{static_cast<const uint8_t *>(tags), seq, uint32_t(i), 0}, st, chain);
            if (rc != HXT_OK) return rc;
            continue;
        }
        rc = s_send ? run_copy<false, true>(pl, src, buf, s_send, st, chain)
                    : run_copy<false, false>(pl, src, buf, nullptr, st, chain);
        if (rc != HXT_OK) return rc;
        rc = s_recv ? run_copy<true, true>(pl, x.dst + i * T, buf, s_recv, st, chain)
                    : run_copy<true, false>(pl, x.dst + i * T, buf, nullptr, st, chain);
        if (rc != HXT_OK) return rc;
    }
    std::vector<hipEvent_t> done;
    if (!borrow_events(pl, 2, done)) return HXT_EHIP;
    hipError_t e = hipEventRecord(done[0], a);
    if (e == hipSuccess) e = hipEventRecord(done[1], b);
    if (e == hipSuccess) e = hipStreamWaitEvent(b, done[0], 0);
    if (e == hipSuccess) e = hipStreamWaitEvent(a, done[1], 0);
    if (e == hipSuccess && third != a && third != b) {
        e = hipStreamWaitEvent(third, done[0], 0);
        if (e == hipSuccess) e = hipStreamWaitEvent(third, done[1], 0);
    }
    return_events(pl, done);
    return e == hipSuccess ? HXT_OK : hip_fail(e);
}

}  // namespace

// ---- C ABI ---------------------------------------------------------------------------

extern "C" {

int hxt_plan_multi(const hxt_tensor_desc_t *tensors, int n_tensors, int n_lanes, size_t chunk_bytes,
                   hxt_plan_t **out)
{
    if (!out) return HXT_EINVAL;
    hxt_plan_t *pl = new (std::nothrow) hxt_plan_t;
    if (!pl) return HXT_ENOMEM;
    int rc;
    try {
        rc = build_plan(tensors, n_tensors, n_lanes, chunk_bytes,
                        uint32_t(env_int("HXT_TILE_BYTES", int(kDefaultTileBytes))), pl->p);
        if (rc == HXT_OK) rc = upload(*pl);
    } catch (const std::bad_alloc &) {
        rc = HXT_ENOMEM;
    }
    if (rc != HXT_OK) {
        hxt_plan_destroy(pl);
        return rc;
    }
    *out = pl;
    return HXT_OK;
}

int hxt_plan(const int64_t *shape, const int64_t *strides, int ndim, hxt_dtype_t dtype, int n_lanes,
             size_t chunk_bytes, hxt_plan_t **out)
{
    hxt_tensor_desc_t d{ndim, shape, strides, dtype};
    return hxt_plan_multi(&d, 1, n_lanes, chunk_bytes, out);
}

int hxt_plan_destroy(hxt_plan_t *plan)
{
    if (!plan) return HXT_OK;
    int rc = HXT_OK;
    auto release = [&](void *p) {
        if (p && hipFree(p) != hipSuccess) rc = HXT_EHIP;
    };
    release(plan->d_tiles);
    release(plan->d_chunk_tiles);
    release(plan->d_tensors);
    release(plan->d_inc);
    for (OpState &o : plan->ops) {
        release(o.acc);
        if (o.ev && hipEventDestroy(o.ev) != hipSuccess) rc = HXT_EHIP;
    }
    for (hipEvent_t e : plan->ev_free)
        if (hipEventDestroy(e) != hipSuccess) rc = HXT_EHIP;
    delete plan;
    return rc;
}

int hxt_plan_set_option(hxt_plan_t *plan, int option, int value)
{
    if (!plan) return HXT_EINVAL;
    switch (option) {
    case HXT_OPT_PACKED_HINT:
        if (value < -1 || value > 1) return HXT_EINVAL;
        plan->nt_packed = value;
        return HXT_OK;
    case HXT_OPT_STAGE_D2H:
        if (value < 0 || value > 1) return HXT_EINVAL;
        plan->stage_d2h_kernel = value;
        return HXT_OK;
    }
    return HXT_EINVAL;
}

size_t hxt_plan_message_bytes(const hxt_plan_t *plan) { return plan ? plan->p.N : 0; }
size_t hxt_plan_stream_bytes(const hxt_plan_t *plan) { return plan ? plan->p.L : 0; }
size_t hxt_plan_packed_bytes(const hxt_plan_t *plan) { return plan ? plan->p.C * plan->p.B : 0; }
size_t hxt_plan_chunk_bytes(const hxt_plan_t *plan) { return plan ? plan->p.B : 0; }
int hxt_plan_num_chunks(const hxt_plan_t *plan) { return plan ? int(plan->p.C) : 0; }
int hxt_plan_num_lanes(const hxt_plan_t *plan) { return plan ? plan->p.k : 0; }
int hxt_plan_num_tensors(const hxt_plan_t *plan) { return plan ? int(plan->p.tensors.size()) : 0; }

int hxt_plan_chunk_info(const hxt_plan_t *plan, int c, hxt_chunk_info_t *out)
{
    if (!plan || !out || c < 0 || uint64_t(c) >= plan->p.C) return HXT_EINVAL;
    const Plan &p = plan->p;
    const uint64_t lo = uint64_t(c) * p.B, hi = lo + p.chunk_padded(c);
    uint64_t payload = 0;
    for (const TensorPlan &t : p.tensors) {
        const uint64_t a = std::max(lo, t.stream_off), b = std::min(hi, t.stream_off + t.bytes);
        if (b > a) payload += b - a;
    }
    out->lane = int32_t(uint64_t(c) % p.k);
    out->slot = int32_t(uint64_t(c) / p.k);
    out->stream_off = lo;
    out->padded = hi - lo;
    out->payload = payload;
    out->packed_off = p.chunk_packed_off(c);
    return HXT_OK;
}

int hxt_plan_lane_info(const hxt_plan_t *plan, int lane, hxt_lane_info_t *out)
{
    if (!plan || !out || lane < 0 || lane >= plan->p.k) return HXT_EINVAL;
    uint64_t r[2][2] = {{0, 0}, {0, 0}};
    stage_ranges(plan->p, lane, r);
    out->packed_off = plan->p.lane_off[lane];
    out->bytes = r[0][1];
    out->n_chunks = int32_t(plan->p.lane_chunks[lane]);
    return HXT_OK;
}

int hxt_plan_tensor_unpack_safe(const hxt_plan_t *plan, int t)
{
    if (!plan || t < 0 || size_t(t) >= plan->p.tensors.size()) return HXT_EINVAL;
    return plan->p.tensors[t].unpack_safe ? 1 : 0;
}

int hxt_plan_tensor_kind(const hxt_plan_t *plan, int t)
{
    if (!plan || t < 0 || size_t(t) >= plan->p.tensors.size()) return HXT_EINVAL;
    return int(plan->p.tensors[t].kind);
}

int hxt_pack(const hxt_plan_t *plan, const void *const *src, void *packed, uint64_t *sums, void *stream)
{
    int rc = check_common(plan, packed);
    if (rc != HXT_OK || plan->p.C == 0) return rc;
    void *const *ptrs = const_cast<void *const *>(src);
    if ((rc = check_tensor_pointers(plan->p, ptrs)) != HXT_OK) return rc;
    hxt_plan_t &pl = *const_cast<hxt_plan_t *>(plan);     // only the slot bookkeeping is mutable
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint8_t *pk = static_cast<uint8_t *>(packed);
    return sums ? run_copy<false, true>(pl, ptrs, pk, sums, st) : run_copy<false, false>(pl, ptrs, pk, nullptr, st);
}

int hxt_unpack(const hxt_plan_t *plan, const void *packed, void *const *dst, uint64_t *sums, void *stream)
{
    int rc = check_common(plan, packed);
    if (rc != HXT_OK || plan->p.C == 0) return rc;
    if ((rc = check_tensor_pointers(plan->p, dst)) != HXT_OK) return rc;
    if (!plan->p.all_unpack_safe) return HXT_EOVERLAP;
    hxt_plan_t &pl = *const_cast<hxt_plan_t *>(plan);
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint8_t *pk = const_cast<uint8_t *>(static_cast<const uint8_t *>(packed));
    return sums ? run_copy<true, true>(pl, dst, pk, sums, st) : run_copy<true, false>(pl, dst, pk, nullptr, st);
}

int hxt_pack_batch(int n, const hxt_plan_t *const *plans, const void *const *const *src, void *const *packed,
                   uint64_t *const *sums, void *stream)
{
    return run_batch<false>(n, plans, const_cast<void *const *const *>(src), packed, sums,
                            static_cast<hipStream_t>(stream));
}

int hxt_unpack_batch(int n, const hxt_plan_t *const *plans, const void *const *packed, void *const *const *dst,
                     uint64_t *const *sums, void *stream)
{
    return run_batch<true>(n, plans, dst, const_cast<void *const *>(packed), sums, static_cast<hipStream_t>(stream));
}

int hxt_host_forward(const hxt_plan_t *plan, int lane, const void *from, void *to, int n_threads)
{
    if (!plan) return HXT_EINVAL;
    const Plan &p = plan->p;
    if (lane < -1 || lane >= p.k) return HXT_EINVAL;
    if (p.C == 0) return HXT_OK;
    if (!from || !to) return HXT_EINVAL;
    const int first = lane < 0 ? 0 : lane;                       // lanes first .. first + n_lanes - 1
    const size_t n_lanes = lane < 0 ? size_t(p.k) : 1;
    auto copy_lane = [&](int l) {
        uint64_t r[2][2];
        if (stage_ranges(p, l, r))
            std::memcpy(static_cast<uint8_t *>(to) + r[0][0], static_cast<const uint8_t *>(from) + r[0][0], r[0][1]);
    };
    const size_t workers = std::min<size_t>(n_lanes, n_threads < 1 ? n_lanes : size_t(n_threads));
    if (workers <= 1) {
        for (size_t i = 0; i < n_lanes; ++i) copy_lane(first + int(i));
        return HXT_OK;
    }
    // A worker takes lanes w, w + workers, ...  If a thread cannot be created, the threads that did start
    // are joined and the lanes of the missing workers are copied here: the copy still completes.
    std::thread pool[64];
    const size_t n_pool = std::min<size_t>(workers, 64);
    auto work = [&](size_t w) {
        for (size_t i = w; i < n_lanes; i += n_pool) copy_lane(first + int(i));
    };
    size_t started = 0;
    try {
        for (; started + 1 < n_pool; ++started) pool[started] = std::thread(work, started + 1);
    } catch (...) {
    }
    work(0);                                         // the calling thread is worker 0
    for (size_t w = 0; w < started; ++w) pool[w].join();
    for (size_t w = started + 1; w < n_pool; ++w) work(w);      // workers that never started
    return HXT_OK;
}

namespace {
struct HopJob {
    const hxt_plan_t *plan;
    int lane;
    const void *from;
    void *to;
    int n_threads;
};
void run_hop(void *arg)
{
    HopJob *j = static_cast<HopJob *>(arg);
    (void)hxt_host_forward(j->plan, j->lane, j->from, j->to, j->n_threads);
    delete j;
}
}  // namespace

int hxt_stage_hop(const hxt_plan_t *plan, int lane, const void *from_pinned, void *to_pinned, int n_threads,
                  void *stream)
{
    if (!plan || lane < -1 || lane >= plan->p.k) return HXT_EINVAL;
    if (plan->p.C == 0) return HXT_OK;
    if (!from_pinned || !to_pinned) return HXT_EINVAL;
    HopJob *j = new (std::nothrow) HopJob{plan, lane, from_pinned, to_pinned, n_threads};
    if (!j) return HXT_ENOMEM;
    hipError_t e = hipLaunchHostFunc(static_cast<hipStream_t>(stream), run_hop, j);
    if (e != hipSuccess) {
        delete j;
        return hip_fail(e);
    }
    return HXT_OK;
}

int hxt_unpack_accumulate(const hxt_plan_t *plan, const void *packed, void *const *dst, uint64_t *sums,
                          void *stream)
{
    int rc = check_common(plan, packed);
    if (rc != HXT_OK || plan->p.C == 0) return rc;
    if ((rc = check_tensor_pointers(plan->p, dst)) != HXT_OK) return rc;
    const Plan &p = plan->p;
    if (!p.can_accumulate) return HXT_EUNSUPPORTED;
    hxt_plan_t &pl = *const_cast<hxt_plan_t *>(plan);
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint8_t *pk = const_cast<uint8_t *>(static_cast<const uint8_t *>(packed));
    return sums ? run_accumulate<true>(pl, dst, pk, sums, st) : run_accumulate<false>(pl, dst, pk, nullptr, st);
}

// Batched receive-and-accumulate: messages that are one contiguous 16-byte aligned tensor share launches of
// up to kMaxBatch (same checksum choice within a launch); the rest go one by one.
int hxt_unpack_accumulate_batch(int n, const hxt_plan_t *const *plans, const void *const *packed,
                                void *const *const *dst, uint64_t *const *sums, void *stream)
{
    if (n < 0 || (n > 0 && (!plans || !dst || !packed))) return HXT_EINVAL;
    for (int i = 0; i < n; ++i) {                      // validate everything before enqueuing anything
        int rc = check_common(plans[i], packed[i]);
        if (rc != HXT_OK) return rc;
        if (plans[i]->p.C == 0) continue;
        if ((rc = check_tensor_pointers(plans[i]->p, dst[i])) != HXT_OK) return rc;
        if (!plans[i]->p.can_accumulate) return HXT_EUNSUPPORTED;
        for (int j = 0; j < i; ++j)
            if (plans[j] == plans[i] && sums && sums[i] && sums[j]) return HXT_EINVAL;   // one accumulator set per plan
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    BatchLock lock(plans, n);
    int i = 0;
    while (i < n) {
        hxt_plan_t &pl = *const_cast<hxt_plan_t *>(plans[i]);
        const Plan &p = pl.p;
        uint64_t *sm = sums ? sums[i] : nullptr;
        auto fusable = [&](int j) {
            const Plan &q = plans[j]->p;
            return q.C != 0 && q.uniform && reinterpret_cast<uintptr_t>(dst[j][q.uniform_tensor]) % 16 == 0 &&
                   ((sums ? sums[j] : nullptr) != nullptr) == (sm != nullptr);
        };
        if (p.C == 0) {
            ++i;
            continue;
        }
        if (!fusable(i)) {
            uint8_t *pk = const_cast<uint8_t *>(static_cast<const uint8_t *>(packed[i]));
            int rc = sm ? run_accumulate<true>(pl, dst[i], pk, sm, st) : run_accumulate<false>(pl, dst[i], pk, nullptr, st);
            if (rc != HXT_OK) return rc;
            ++i;
            continue;
        }
        UniformArgs a;
        std::memset(&a, 0, sizeof a);
        uint64_t tiles = 0, bytes = 0;
        int j = i;
        while (j < n && a.n < uint32_t(kMaxBatch) && fusable(j) && tiles + plans[j]->p.geom.ntiles < (uint64_t(1) << 31)) {
            hxt_plan_t &pj = *const_cast<hxt_plan_t *>(plans[j]);
            SumCtx cx{nullptr, nullptr, 0, 0, 1, 0};
            if (sm) {
                int rc = claim_slots(pj, OP_UNPACK, st, cx, sums[j]);
                if (rc != HXT_OK) return rc;
                cx.sum_bits = pj.sum_bits_geom;
            }
            const TensorPlan &tp = pj.p.tensors[pj.p.uniform_tensor];
            // `unpack` carries the element kind here: 1 = f32, 0 = bf16
            a.it[a.n++] = UniformItem{pj.p.geom, static_cast<uint8_t *>(dst[j][pj.p.uniform_tensor]),
                                      const_cast<uint8_t *>(static_cast<const uint8_t *>(packed[j])), cx, uint32_t(tiles),
                                      tp.dtype == HXT_F32 ? 1u : 0u};
            tiles += pj.p.geom.ntiles;
            bytes += pj.p.C * pj.p.B;
            ++j;
        }
        const bool ntp = plans[i]->nt_packed >= 0 ? plans[i]->nt_packed != 0 : packed_nontemporal(bytes);
        with_hints(ntp, [&]<bool NTU, bool NTP>() {
            if (sm) k_uniform_accumulate<true, NTU, NTP><<<uint32_t(tiles), kThreads, 0, st>>>(a);
            else k_uniform_accumulate<false, NTU, NTP><<<uint32_t(tiles), kThreads, 0, st>>>(a);
        });
        HXT_HIP(hipGetLastError());
        i = j;
    }
    return HXT_OK;
}

int hxt_exchange_stream(const hxt_plan_t *plan, const hxt_exchange_t *x)
{
    if (!plan || !x || x->n_messages < 0 || x->n_buffers < 1) return HXT_EINVAL;
    if (x->path != HXT_DEVICE_DIRECT && x->path != HXT_CPU_FORWARD) return HXT_EINVAL;
    const Plan &p = plan->p;
    if (x->n_messages == 0 || p.C == 0) return HXT_OK;
    const bool fwd = x->path == HXT_CPU_FORWARD;
    if (!x->src || !x->dst || !x->packed_send || (fwd && (!x->packed_recv || !x->host_pinned))) return HXT_EINVAL;
    const size_t T = p.tensors.size();
    int rc;
    for (int b = 0; b < x->n_buffers; ++b) {                  // validate before anything is enqueued
        if ((rc = check_common(plan, x->packed_send[b])) != HXT_OK) return rc;
        if (fwd) {
            if ((rc = check_common(plan, x->packed_recv[b])) != HXT_OK) return rc;
            if (!x->host_pinned[b]) return HXT_EINVAL;
            if (reinterpret_cast<uintptr_t>(x->host_pinned[b]) % HXT_ALIGN) return HXT_EALIGN;
        }
    }
    const bool tagged = x->tags_send != nullptr;
    if (tagged) {
        if (!x->status || x->send_sums || x->recv_sums || (fwd && (!x->tags_recv || !x->tags_pinned))) return HXT_EINVAL;
        if (reinterpret_cast<uintptr_t>(x->status) % 4) return HXT_EALIGN;
        for (int b = 0; b < x->n_buffers; ++b) {
            if (!x->tags_send[b] || (fwd && (!x->tags_recv[b] || !x->tags_pinned[b]))) return HXT_EINVAL;
            if (reinterpret_cast<uintptr_t>(x->tags_send[b]) % 16 ||
                (fwd && (reinterpret_cast<uintptr_t>(x->tags_recv[b]) % 16 || reinterpret_cast<uintptr_t>(x->tags_pinned[b]) % 16)))
                return HXT_EALIGN;
        }
    }
    if (!p.all_unpack_safe) return HXT_EOVERLAP;
    for (int i = 0; i < x->n_messages; ++i) {
        if ((rc = check_tensor_pointers(p, const_cast<void *const *>(x->src + i * T))) != HXT_OK) return rc;
        if ((rc = check_tensor_pointers(p, x->dst + i * T)) != HXT_OK) return rc;
    }
    hipStream_t sp = static_cast<hipStream_t>(x->stream_pack), ss = static_cast<hipStream_t>(x->stream_stage),
                su = static_cast<hipStream_t>(x->stream_unpack);
    if (x->drain_every < 0 || x->direct_mode < HXT_DIRECT_AUTO || x->direct_mode > HXT_DIRECT_EVENTS) return HXT_EINVAL;
    if (!fwd) {
        const bool chains_ok = x->n_buffers % 2 == 0 && sp != su;
        bool fused_ok = !tagged && x->n_buffers >= 2 && p.uniform && !x->send_sums == !x->recv_sums;
        for (int i = 0; fused_ok && i < x->n_messages; ++i)
            fused_ok = reinterpret_cast<uintptr_t>(x->src[i * T + p.uniform_tensor]) % 16 == 0 &&
                       reinterpret_cast<uintptr_t>(x->dst[i * T + p.uniform_tensor]) % 16 == 0;
        int mode = x->direct_mode;
        if (mode == HXT_DIRECT_AUTO) mode = chains_ok ? HXT_DIRECT_TWO_CHAINS : (fused_ok ? HXT_DIRECT_FUSED : HXT_DIRECT_EVENTS);
        if (mode == HXT_DIRECT_TWO_CHAINS) {
            if (!chains_ok) return HXT_EINVAL;
            return chained_direct_stream(*const_cast<hxt_plan_t *>(plan), *x, sp, su, ss);
        }
        if (mode == HXT_DIRECT_FUSED) {
            if (!fused_ok) return HXT_EINVAL;
            return fused_direct_stream(*const_cast<hxt_plan_t *>(plan), *x, sp, ss, su);
        }
    }
    // per buffer set: packed (pack done), drained (send buffer may be rewritten), staged (host copy
    // complete), landed (host buffer may be rewritten), tags read (pinned tag buffer may be rewritten)
    enum { PACKED, DRAINED, STAGED, LANDED, TAGS_READ, KINDS };
    const int nb = x->n_buffers;
    hxt_plan_t &pl = *const_cast<hxt_plan_t *>(plan);
    std::vector<hipEvent_t> ev;
    if (!borrow_events(pl, size_t(nb) * KINDS, ev)) return HXT_EHIP;
    auto at = [&](int kind, int b) -> hipEvent_t & { return ev[size_t(b) * KINDS + kind]; };
    auto cleanup = [&]() { return_events(pl, ev); };
    rc = HXT_OK;
    auto hip = [&](hipError_t e) {
        if (e != hipSuccess && rc == HXT_OK) rc = hip_fail(e);
        return e == hipSuccess;
    };
    const uint32_t tag_vecs = uint32_t(p.C * (sizeof(hxt_chunk_tag_t) / 16));
    auto copy_tags = [&](void *to, const void *from, hipStream_t st) {
        k_copy_tags<<<std::min<uint32_t>((tag_vecs + kThreads - 1) / kThreads, 64u), kThreads, 0, st>>>(
            static_cast<u32x4 *>(to), static_cast<const u32x4 *>(from), tag_vecs);
        return hip(hipGetLastError());
    };
    const int drain_every = x->drain_every;
    for (int i = 0; i < x->n_messages && rc == HXT_OK; ++i) {
        const int b = i % nb;
        uint64_t *s_send = x->send_sums ? x->send_sums + size_t(i) * p.C : nullptr;
        uint64_t *s_recv = x->recv_sums ? x->recv_sums + size_t(i) * p.C : nullptr;
        const uint64_t seq = x->seq_base + uint64_t(i);
        if (i >= nb && !hip(hipStreamWaitEvent(sp, at(DRAINED, b), 0))) break;
        if (i >= nb && fwd && tagged && !hip(hipStreamWaitEvent(sp, at(TAGS_READ, b), 0))) break;
        rc = tagged ? hxt_pack_seal(plan, x->src + i * T, x->packed_send[b], seq, uint32_t(i),
                                    static_cast<hxt_chunk_tag_t *>(x->tags_send[b]), sp)
                    : hxt_pack(plan, x->src + i * T, x->packed_send[b], s_send, sp);
        if (rc != HXT_OK) break;
        // The tags go to the pinned buffer from the pack stream, by a small kernel, so that the staging stream
        // carries nothing but the large device-to-host copies.
        if (fwd && tagged && !copy_tags(x->tags_pinned[b], x->tags_send[b], sp)) break;
        if (!hip(hipEventRecord(at(PACKED, b), sp))) break;
        const void *arrived = x->packed_send[b];
        const void *arrived_tags = tagged ? x->tags_send[b] : nullptr;
        if (fwd) {
            if (!hip(hipStreamWaitEvent(ss, at(PACKED, b), 0))) break;
            if (i >= nb && !hip(hipStreamWaitEvent(ss, at(LANDED, b), 0))) break;
            if ((rc = hxt_stage_d2h(plan, -1, x->packed_send[b], x->host_pinned[b], ss)) != HXT_OK) break;
            if (!hip(hipEventRecord(at(STAGED, b), ss))) break;
            if (!hip(hipEventRecord(at(DRAINED, b), ss))) break;
            if (!hip(hipStreamWaitEvent(su, at(STAGED, b), 0))) break;
            if ((rc = hxt_stage_h2d(plan, -1, x->host_pinned[b], x->packed_recv[b], su)) != HXT_OK) break;
            if (!hip(hipEventRecord(at(LANDED, b), su))) break;       // straight after the copy: the next device-to-host copy waits on it
            if (tagged && (!copy_tags(x->tags_recv[b], x->tags_pinned[b], su) || !hip(hipEventRecord(at(TAGS_READ, b), su)))) break;
            arrived = x->packed_recv[b];
            if (tagged) arrived_tags = x->tags_recv[b];
        } else {
            if (!hip(hipStreamWaitEvent(su, at(PACKED, b), 0))) break;
        }
        rc = tagged ? hxt_unpack_verify(plan, arrived, static_cast<const hxt_chunk_tag_t *>(arrived_tags), seq, uint32_t(i),
                                        x->dst + i * T, x->status + size_t(i) * (p.C + 1), su)
                    : hxt_unpack(plan, arrived, x->dst + i * T, s_recv, su);
        if (rc != HXT_OK) break;
        if (!fwd && !hip(hipEventRecord(at(DRAINED, b), su))) break;
        // CPU forwarding, on request only: with more than about 16 messages' worth of copies and event waits
        // outstanding the runtime stops overlapping the two copy directions (measured: 760 us per 32 MiB
        // message up to 16 enqueued, 1300-1900 us beyond; waiting on an older message's event does not help,
        // an empty queue does), so a caller may have the three streams drained every few messages.
        if (fwd && drain_every > 0 && (i + 1) % drain_every == 0 && i + 1 < x->n_messages)
            if (!hip(hipStreamSynchronize(su)) || !hip(hipStreamSynchronize(ss)) || !hip(hipStreamSynchronize(sp))) break;
    }
    cleanup();
    return rc;
}

// hxt_pack for a message that is one contiguous tensor, with no plan and no allocation: the geometry is
// closed form (host arithmetic on the stack) and the checksum accumulators live in this GPU's `scratch`.
int hxt_pack_noalloc(const void *src, size_t message_bytes, int n_lanes, size_t chunk_bytes, void *packed,
                     uint64_t *sums, void *stream)
{
    if (n_lanes < 1 || n_lanes > 1024 || chunk_bytes == 0 || chunk_bytes % HXT_ALIGN) return HXT_EINVAL;
    if (message_bytes > (uint64_t(1) << 40)) return HXT_EUNSUPPORTED;
    if (message_bytes == 0) return HXT_OK;
    if (!src || !packed) return HXT_EINVAL;
    if (reinterpret_cast<uintptr_t>(packed) % HXT_ALIGN) return HXT_EALIGN;
    const uint32_t tile = uint32_t(env_int("HXT_TILE_BYTES", int(kDefaultTileBytes)));
    if (tile == 0 || tile % HXT_ALIGN || tile > (1u << 24)) return HXT_EINVAL;
    const uint64_t L = (uint64_t(message_bytes) + HXT_ALIGN - 1) / HXT_ALIGN * HXT_ALIGN;
    UniformArgs a;
    std::memset(&a, 0, sizeof a);
    ChunkGeom &g = a.it[0].g;
    int rc = make_geom(message_bytes, L, chunk_bytes, uint32_t(n_lanes), tile, g);
    if (rc != HXT_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    SumCtx cx{nullptr, nullptr, 0, 0, 1, 0};
    if (sums) {
        const uint32_t fan = choose_fan(g.tpc);
        const size_t slots = size_t(g.C) * (fan + 1);
        if (slots > kScratchSlots) return HXT_EUNSUPPORTED;           // more chunks than the fixed scratch serves
        uint8_t *ptr = nullptr;
        if ((rc = scratch_on_device(&ptr)) != HXT_OK) return rc;
        const bool two_word = env_int("HXT_TWO_WORD_COMMIT", 0) != 0;
        cx = SumCtx{sums, ptr, kScratchSlotStride, two_word ? 0 : single_word_bits(chunk_bytes, max_arrivals(g.tpc, fan)),
                    fan, g.C};
        // The array keeps whatever the last call on this GPU left: the slots this call uses start at zero.
        const uint32_t nvec = uint32_t(slots * kScratchSlotStride / 16);
        k_fill_zero<<<std::min<uint32_t>((nvec + kThreads - 1) / kThreads, 256u), kThreads, 0, st>>>(
            reinterpret_cast<u32x4 *>(ptr), nvec);
        HXT_HIP(hipGetLastError());
    }
    uint8_t *user = const_cast<uint8_t *>(static_cast<const uint8_t *>(src));
    a.n = 1;
    a.it[0].user = user;
    a.it[0].packed = static_cast<uint8_t *>(packed);
    a.it[0].cx = cx;
    a.it[0].first_tile = 0;
    a.it[0].unpack = 0;
    const bool ntp = packed_nontemporal(uint64_t(g.C) * g.B);
    if (reinterpret_cast<uintptr_t>(user) % 16 == 0) {
        if (sums) launch_uniform<DIR_PACK, true>(a, g.ntiles, ntp, st);
        else launch_uniform<DIR_PACK, false>(a, g.ntiles, ntp, st);
    } else if (sums) {
        k_uniform_any<false, true><<<g.ntiles, kThreads, 0, st>>>(a);
    } else {
        k_uniform_any<false, false><<<g.ntiles, kThreads, 0, st>>>(a);
    }
    HXT_HIP(hipGetLastError());
    return HXT_OK;
}

int hxt_checksum(const hxt_plan_t *plan, const void *packed, uint64_t *sums, void *stream)
{
    int rc = check_common(plan, packed);
    if (rc != HXT_OK || plan->p.C == 0) return rc;
    if (!sums) return HXT_EINVAL;
    hxt_plan_t &pl = *const_cast<hxt_plan_t *>(plan);
    hipStream_t st = static_cast<hipStream_t>(stream);
    SumCtx cx{nullptr, nullptr, 0, 0, 1, 0};
    SlotsLock lock(pl.slots_mu);
    if ((rc = claim_slots(pl, OP_CHECKSUM, st, cx, sums)) != HXT_OK) return rc;
    cx.sum_bits = pl.sum_bits_geom;
    const uint8_t *pk = static_cast<const uint8_t *>(packed);
    if (packed_nontemporal(pl))
        k_checksum<true><<<pl.p.geom.ntiles, kThreads, 0, st>>>(pl.p.geom, pk, cx);
    else
        k_checksum<false><<<pl.p.geom.ntiles, kThreads, 0, st>>>(pl.p.geom, pk, cx);
    HXT_HIP(hipGetLastError());
    return HXT_OK;
}



int hxt_pack_seal(const hxt_plan_t *plan, const void *const *src, void *packed, uint64_t seq, uint32_t micro_batch,
                  hxt_chunk_tag_t *tags, void *stream)
{
    if (plan && plan->p.C == 0) return HXT_OK;
    return run_copy_tag<false>(plan, const_cast<void *const *>(src), packed, tags, TagWork{nullptr, seq, micro_batch, 0},
                               stream);
}

int hxt_unpack_verify(const hxt_plan_t *plan, const void *packed, const hxt_chunk_tag_t *tags, uint64_t seq,
                      uint32_t micro_batch, void *const *dst, uint32_t *status, void *stream)
{
    if (plan && plan->p.C == 0) return hxt_verify(plan, packed, tags, seq, micro_batch, status, stream);
    return run_copy_tag<true>(plan, dst, const_cast<void *>(packed), status,
                              TagWork{reinterpret_cast<const uint8_t *>(tags), seq, micro_batch, 0}, stream);
}

int hxt_pack_seal_batch(int n, const hxt_plan_t *const *plans, const void *const *const *src, void *const *packed,
                        const uint64_t *seq, const uint32_t *micro_batch, hxt_chunk_tag_t *const *tags, void *stream)
{
    return run_tag_batch<false>(n, plans, const_cast<void *const *const *>(src), packed,
                                reinterpret_cast<void *const *>(tags), nullptr, seq, micro_batch,
                                static_cast<hipStream_t>(stream));
}

int hxt_unpack_verify_batch(int n, const hxt_plan_t *const *plans, const void *const *packed,
                            const hxt_chunk_tag_t *const *tags, const uint64_t *seq, const uint32_t *micro_batch,
                            void *const *const *dst, uint32_t *const *status, void *stream)
{
    return run_tag_batch<true>(n, plans, dst, const_cast<void *const *>(packed), reinterpret_cast<void *const *>(status),
                               tags, seq, micro_batch, static_cast<hipStream_t>(stream));
}

int hxt_checksum2(const hxt_plan_t *plan, const void *packed, uint64_t *sums2, void *stream)
{
    if (plan && plan->p.C == 0) return HXT_OK;
    return run_sum2(plan, packed, SUM2_SUMS, sums2, TagWork{nullptr, 0, 0, 0}, stream);
}

int hxt_seal(const hxt_plan_t *plan, const void *packed, uint64_t seq, uint32_t micro_batch, hxt_chunk_tag_t *tags,
             void *stream)
{
    if (plan && plan->p.C == 0) return HXT_OK;
    return run_sum2(plan, packed, SUM2_SEAL, tags, TagWork{nullptr, seq, micro_batch, 0}, stream);
}

int hxt_verify(const hxt_plan_t *plan, const void *packed, const hxt_chunk_tag_t *tags, uint64_t seq,
               uint32_t micro_batch, uint32_t *status, void *stream)
{
    if (!plan || !status) return HXT_EINVAL;
    if (plan->p.C == 0) {                       // nothing to check: status[0] = 0 rejected chunks
        if (plan->device < 0) {
            g_last_hip = int(hipErrorNoDevice);
            return HXT_EHIP;
        }
        k_count_rejected<<<1, kThreads, 0, static_cast<hipStream_t>(stream)>>>(status, 0);
        HXT_HIP(hipGetLastError());
        return HXT_OK;
    }
    return run_sum2(plan, packed, SUM2_VERIFY, status,
                    TagWork{reinterpret_cast<const uint8_t *>(tags), seq, micro_batch, 0}, stream);
}

int hxt_stage_d2h(const hxt_plan_t *plan, int lane, const void *packed_dev, void *host_pinned, void *stream)
{
    return stage(plan, lane, 0, -1, packed_dev, host_pinned, hipMemcpyDeviceToHost, stream);
}

int hxt_stage_h2d(const hxt_plan_t *plan, int lane, const void *host_pinned, void *packed_dev, void *stream)
{
    return stage(plan, lane, 0, -1, host_pinned, packed_dev, hipMemcpyHostToDevice, stream);
}

int hxt_stage_d2h_slots(const hxt_plan_t *plan, int lane, int first_slot, int n_slots, const void *packed_dev,
                        void *host_pinned, void *stream)
{
    if (n_slots < 0) return HXT_EINVAL;
    return stage(plan, lane, first_slot, n_slots, packed_dev, host_pinned, hipMemcpyDeviceToHost, stream);
}

int hxt_stage_h2d_slots(const hxt_plan_t *plan, int lane, int first_slot, int n_slots, const void *host_pinned,
                        void *packed_dev, void *stream)
{
    if (n_slots < 0) return HXT_EINVAL;
    return stage(plan, lane, first_slot, n_slots, host_pinned, packed_dev, hipMemcpyHostToDevice, stream);
}

const char *hxt_strerror(int status)
{
    switch (status) {
    case HXT_OK: return "ok";
    case HXT_EINVAL: return "invalid argument";
    case HXT_EALIGN: return "pointer alignment";
    case HXT_EUNSUPPORTED: return "unsupported size";
    case HXT_EOVERLAP: return "destination view may alias itself";
    case HXT_EHIP: return "HIP runtime error (or no device table: plan was created without a GPU)";
    case HXT_ENOMEM: return "out of memory";
    }
    return "unknown status";
}

int hxt_last_hip_error(void) { return g_last_hip; }

const char *hxt_version(void) { return "hxt 0.4 (gfx950)"; }

}  // extern "C"
