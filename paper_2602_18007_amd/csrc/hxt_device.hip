// HIP kernels (gfx950) and the C ABI of libhxt.
//
// Data plane of the paper's Section 2.2 transfer: user buffer -> chunk buffer on
// the sender (pack), chunk buffer -> user buffer on the receiver (unpack), plus
// the explicit device<->host copies of the CPU-forwarding variant (Section 2.1)
// and a per-chunk integrity sum.  Every kernel is a pure byte mover: data is
// handled as unsigned integers so that any bit pattern survives unchanged.
//
// Work decomposition: the host planner cuts the message into tiles (one per
// workgroup, never crossing a chunk or a tensor); a workgroup reads its 64-byte
// tile record with scalar loads and moves the bytes with 128-bit vector
// accesses.  Checksums are accumulated per thread in 64-bit integers, reduced
// across the 64-lane wavefront with shuffles, across the four waves through
// LDS, and added to the chunk's total with one 64-bit atomic per workgroup;
// integer addition makes the result independent of the order of arrival.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>

#include "hxt_internal.h"

using namespace hxt;

namespace {

constexpr int kThreads = 256;

struct BasePtrs {
    uint8_t *p[kMaxGroupTensors];
};

// ---- small device helpers ----------------------------------------------------

template <bool NT>
__device__ __forceinline__ uint4 load16(const uint4 *p)
{
    if constexpr (NT) {
        return uint4{__builtin_nontemporal_load(&p->x), __builtin_nontemporal_load(&p->y),
                     __builtin_nontemporal_load(&p->z), __builtin_nontemporal_load(&p->w)};
    } else {
        return *p;
    }
}

template <bool NT>
__device__ __forceinline__ void store16(uint4 *p, uint4 v)
{
    if constexpr (NT) {
        __builtin_nontemporal_store(v.x, &p->x);
        __builtin_nontemporal_store(v.y, &p->y);
        __builtin_nontemporal_store(v.z, &p->z);
        __builtin_nontemporal_store(v.w, &p->w);
    } else {
        *p = v;
    }
}

__device__ __forceinline__ uint64_t words_sum(uint4 v)
{
    return (uint64_t(v.x) + uint64_t(v.y)) + (uint64_t(v.z) + uint64_t(v.w));
}

__device__ __forceinline__ uint32_t fast_div(uint32_t n, FastDiv d)
{
    return uint32_t((uint64_t(n) * d.mul) >> (31 + d.shift));
}

// Sum over the workgroup, then one atomic into the chunk's total.
__device__ __forceinline__ void block_add(uint64_t acc, uint64_t *dst)
{
    __shared__ uint64_t part[kThreads / 64];
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_down(acc, o, 64);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) part[wave] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint64_t s = 0;
#pragma unroll
        for (int w = 0; w < kThreads / 64; ++w) s += part[w];
        atomicAdd(reinterpret_cast<unsigned long long *>(dst), static_cast<unsigned long long>(s));
    }
}

// Pad bytes (fewer than 256): pack writes zeros, unpack only reads them for the sum.
template <bool UNPACK, bool CSUM>
__device__ __forceinline__ uint64_t zero_tile(const Tile &t, uint8_t *packed)
{
    uint64_t acc = 0;
    uint8_t *pk = packed + t.packed_off;
    for (uint32_t i = threadIdx.x; i < t.n0; i += kThreads) {
        if constexpr (!UNPACK) pk[i] = 0;
        if constexpr (UNPACK && CSUM) acc += uint64_t(pk[i]) << (8 * ((t.packed_off + i) & 3));
    }
    return acc;
}

__global__ void k_fill_zero(uint64_t *p, uint32_t n)
{
    uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// ---- contiguous tensors: straight 128-bit copy --------------------------------
// Each thread keeps UNROLL independent 16-byte loads in flight before its first store.
template <bool UNPACK, bool CSUM, int UNROLL, bool NT>
__global__ __launch_bounds__(kThreads) void k_contig(const Tile *__restrict__ tiles, BasePtrs bases,
                                                     uint8_t *__restrict__ packed, uint64_t *__restrict__ sums)
{
    const Tile t = tiles[blockIdx.x];
    uint64_t acc = 0;
    if (t.kind == K_ZERO) {
        acc = zero_tile<UNPACK, CSUM>(t, packed);
    } else {
        uint8_t *user = bases.p[t.tensor] + t.src_off;
        uint8_t *pk = packed + t.packed_off;
        const uint4 *s = reinterpret_cast<const uint4 *>(UNPACK ? pk : user);
        uint4 *d = reinterpret_cast<uint4 *>(UNPACK ? user : pk);
        const uint32_t nvec = t.n0 >> 4;
        constexpr uint32_t STEP = kThreads * UNROLL;
        const uint32_t full = nvec / STEP * STEP;            // uniform: blocks that need no bounds checks
        for (uint32_t v = threadIdx.x; v < full; v += STEP) {
            uint4 r[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) r[u] = load16<NT>(s + v + u * kThreads);
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                store16<NT>(d + v + u * kThreads, r[u]);
                if constexpr (CSUM) acc += words_sum(r[u]);
            }
        }
        for (uint32_t v = full + threadIdx.x; v < nvec; v += kThreads) {
            const uint4 r = load16<NT>(s + v);
            store16<NT>(d + v, r);
            if constexpr (CSUM) acc += words_sum(r);
        }
        const uint32_t tail = t.n0 & 15;                 // only the last tile of a tensor
        if (threadIdx.x < tail) {
            const uint32_t i = (nvec << 4) + threadIdx.x;
            const uint8_t b = (UNPACK ? pk : user)[i];
            (UNPACK ? user : pk)[i] = b;
            if constexpr (CSUM) acc += uint64_t(b) << (8 * (i & 3));
        }
    }
    if constexpr (CSUM) block_add(acc, sums + t.chunk);
}

// ---- rows: innermost dimension contiguous, outer dimensions strided -------------
// A 16-byte vector never straddles a run (run length and strides are multiples of 16).
// Logical byte -> (row, column) and row -> outer indices use multiply-shift division.
template <bool UNPACK, bool CSUM, int UNROLL, bool NT>
__global__ __launch_bounds__(kThreads) void k_rows(const Tile *__restrict__ tiles,
                                                   const TensorDev *__restrict__ tensors, uint32_t tensor_base,
                                                   BasePtrs bases, uint8_t *__restrict__ packed,
                                                   uint64_t *__restrict__ sums)
{
    const Tile t = tiles[blockIdx.x];
    const TensorDev &td = tensors[tensor_base + t.tensor];
    uint8_t *user = bases.p[t.tensor];
    uint8_t *pk = packed + t.packed_off;
    const uint32_t row_bytes = td.row_bytes;
    const uint64_t row0 = t.src_off / row_bytes;                    // uniform
    const uint32_t col0 = uint32_t(t.src_off - row0 * row_bytes);
    const int outer = td.ndim - 1;
    const uint32_t nvec = t.n0 >> 4;
    uint64_t acc = 0;
    for (uint32_t v0 = threadIdx.x; v0 < nvec; v0 += kThreads * UNROLL) {
        uint4 r[UNROLL];
        uint64_t off[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const uint32_t v = v0 + u * kThreads;
            const uint32_t x = col0 + (v << 4);
            const uint32_t dr = fast_div(x, td.row_div);
            uint32_t row = uint32_t(row0) + dr;
            uint64_t o = x - dr * row_bytes;
            for (int d = outer - 1; d > 0; --d) {
                const uint32_t q = fast_div(row, td.dim_div[d]);
                o += uint64_t(row - q * uint32_t(td.shape[d])) * uint64_t(td.stride_b[d]);
                row = q;
            }
            o += uint64_t(row) * uint64_t(td.stride_b[0]);
            off[u] = o;
            if (v < nvec) r[u] = load16<NT>(reinterpret_cast<const uint4 *>(UNPACK ? pk + (uint64_t(v) << 4) : user + o));
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const uint32_t v = v0 + u * kThreads;
            if (v < nvec) {
                store16<NT>(reinterpret_cast<uint4 *>(UNPACK ? user + off[u] : pk + (uint64_t(v) << 4)), r[u]);
                if constexpr (CSUM) acc += words_sum(r[u]);
            }
        }
    }
    if constexpr (CSUM) block_add(acc, sums + t.chunk);
}

// ---- transpose: logical inner dimension strided, the one before it contiguous ----
// A tile is ni x nj elements (<= 64 x 64).  Storage is read/written along i, the packed
// stream along j, both coalesced; the swap of roles goes through a padded LDS tile.
template <typename E>
__device__ __forceinline__ uint64_t elem_weighted(E v, uint64_t packed_pos)
{
    if constexpr (sizeof(E) == 8) {
        return uint64_t(uint32_t(v)) + uint64_t(uint32_t(uint64_t(v) >> 32));
    } else {
        return uint64_t(v) << (8 * (packed_pos & 3));
    }
}

template <typename E, bool UNPACK, bool CSUM>
__global__ __launch_bounds__(kThreads) void k_transpose(const Tile *__restrict__ tiles, BasePtrs bases,
                                                        uint8_t *__restrict__ packed, uint64_t *__restrict__ sums)
{
    constexpr uint32_t T = kTransposeTile;
    __shared__ E lds[T][T + 1];
    const Tile t = tiles[blockIdx.x];
    uint8_t *user = bases.p[t.tensor] + t.src_off;
    uint8_t *pk = packed + t.packed_off;
    const uint32_t ni = t.n0, nj = t.n1;
    const uint32_t tx = threadIdx.x & (T - 1), ty = threadIdx.x / T;
    constexpr uint32_t TY = kThreads / T;
    uint64_t acc = 0;
    if constexpr (!UNPACK) {
        if (tx < ni)
            for (uint32_t j = ty; j < nj; j += TY) lds[j][tx] = *reinterpret_cast<const E *>(user + j * t.a + tx * sizeof(E));
        __syncthreads();
        if (tx < nj)
            for (uint32_t i = ty; i < ni; i += TY) {
                const E v = lds[tx][i];
                const uint64_t pos = i * t.b + tx * sizeof(E);
                *reinterpret_cast<E *>(pk + pos) = v;
                if constexpr (CSUM) acc += elem_weighted(v, t.packed_off + pos);
            }
    } else {
        if (tx < nj)
            for (uint32_t i = ty; i < ni; i += TY) {
                const uint64_t pos = i * t.b + tx * sizeof(E);
                const E v = *reinterpret_cast<const E *>(pk + pos);
                lds[tx][i] = v;
                if constexpr (CSUM) acc += elem_weighted(v, t.packed_off + pos);
            }
        __syncthreads();
        if (tx < ni)
            for (uint32_t j = ty; j < nj; j += TY) *reinterpret_cast<E *>(user + j * t.a + tx * sizeof(E)) = lds[j][tx];
    }
    if constexpr (CSUM) block_add(acc, sums + t.chunk);
}

// ---- generic: any strides, one element at a time -------------------------------
// One thread per 16 packed bytes; every element's address is recomputed from its
// logical index.  Slow, and only used for views the other kernels do not take.
template <typename E, bool UNPACK, bool CSUM>
__global__ __launch_bounds__(kThreads) void k_generic(const Tile *__restrict__ tiles,
                                                      const TensorDev *__restrict__ tensors, uint32_t tensor_base,
                                                      BasePtrs bases, uint8_t *__restrict__ packed,
                                                      uint64_t *__restrict__ sums)
{
    const Tile t = tiles[blockIdx.x];
    uint64_t acc = 0;
    if (t.kind == K_ZERO) {
        acc = zero_tile<UNPACK, CSUM>(t, packed);
    } else {
        const TensorDev &td = tensors[tensor_base + t.tensor];
        uint8_t *user = bases.p[t.tensor];
        uint8_t *pk = packed + t.packed_off;
        const uint32_t nel = t.n0 / sizeof(E);
        constexpr uint32_t PER = 16 / sizeof(E);
        const uint64_t e0 = t.src_off / sizeof(E);
        for (uint32_t v = threadIdx.x; v * PER < nel; v += kThreads) {
#pragma unroll
            for (uint32_t j = 0; j < PER; ++j) {
                const uint32_t el = v * PER + j;
                if (el < nel) {
                    uint64_t idx = e0 + el, off = 0;
                    for (int d = td.ndim - 1; d >= 0; --d) {
                        const uint64_t q = idx / uint64_t(td.shape[d]);
                        off += (idx - q * uint64_t(td.shape[d])) * uint64_t(td.stride_b[d]);
                        idx = q;
                    }
                    E *u = reinterpret_cast<E *>(user + off);
                    E *p = reinterpret_cast<E *>(pk) + el;
                    const E val = UNPACK ? *p : *u;
                    if constexpr (UNPACK) *u = val; else *p = val;
                    if constexpr (CSUM) acc += elem_weighted(val, uint64_t(el) * sizeof(E));
                }
            }
        }
    }
    if constexpr (CSUM) block_add(acc, sums + t.chunk);
}

// ---- stand-alone checksum of packed chunks ---------------------------------------
template <int UNROLL, bool NT>
__global__ __launch_bounds__(kThreads) void k_checksum(const Tile *__restrict__ tiles,
                                                       const uint8_t *__restrict__ packed,
                                                       uint64_t *__restrict__ sums)
{
    const Tile t = tiles[blockIdx.x];
    const uint4 *s = reinterpret_cast<const uint4 *>(packed + t.packed_off);
    const uint32_t nvec = t.n0 >> 4;
    uint64_t acc = 0;
    for (uint32_t v = threadIdx.x; v < nvec; v += kThreads * UNROLL) {
        uint4 r[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
            r[u] = (v + u * kThreads < nvec) ? load16<NT>(s + v + u * kThreads) : uint4{0, 0, 0, 0};
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) acc += words_sum(r[u]);
    }
    block_add(acc, sums + t.chunk);
}

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

struct Tuning {
    bool nt;
    Tuning() : nt(env_int("HXT_NONTEMPORAL", 1) != 0) {}
};
const Tuning &tuning()
{
    static Tuning t;
    return t;
}

constexpr int kUnroll = 4;

template <bool UNPACK, bool CSUM>
void launch_contig(const Plan &p, const Group &g, const BasePtrs &b, uint8_t *packed, uint64_t *sums, hipStream_t st)
{
    const Tile *tiles = p.d_tiles + g.first;
    if (tuning().nt)
        k_contig<UNPACK, CSUM, kUnroll, true><<<g.count, kThreads, 0, st>>>(tiles, b, packed, sums);
    else
        k_contig<UNPACK, CSUM, kUnroll, false><<<g.count, kThreads, 0, st>>>(tiles, b, packed, sums);
}

template <bool UNPACK, bool CSUM>
void launch_rows(const Plan &p, const Group &g, const BasePtrs &b, uint8_t *packed, uint64_t *sums, hipStream_t st)
{
    const Tile *tiles = p.d_tiles + g.first;
    if (tuning().nt)
        k_rows<UNPACK, CSUM, kUnroll, true><<<g.count, kThreads, 0, st>>>(tiles, p.d_tensors, g.tensor_base, b, packed, sums);
    else
        k_rows<UNPACK, CSUM, kUnroll, false><<<g.count, kThreads, 0, st>>>(tiles, p.d_tensors, g.tensor_base, b, packed, sums);
}

template <bool UNPACK, bool CSUM>
void launch_transpose(const Plan &p, const Group &g, int esize, const BasePtrs &b, uint8_t *packed, uint64_t *sums,
                      hipStream_t st)
{
    const Tile *tiles = p.d_tiles + g.first;
    switch (esize) {
    case 1: k_transpose<uint8_t, UNPACK, CSUM><<<g.count, kThreads, 0, st>>>(tiles, b, packed, sums); break;
    case 2: k_transpose<uint16_t, UNPACK, CSUM><<<g.count, kThreads, 0, st>>>(tiles, b, packed, sums); break;
    case 4: k_transpose<uint32_t, UNPACK, CSUM><<<g.count, kThreads, 0, st>>>(tiles, b, packed, sums); break;
    default: k_transpose<uint64_t, UNPACK, CSUM><<<g.count, kThreads, 0, st>>>(tiles, b, packed, sums); break;
    }
}

template <bool UNPACK, bool CSUM>
void launch_generic(const Plan &p, uint32_t first, uint32_t count, uint32_t tensor_base, int esize, const BasePtrs &b,
                    uint8_t *packed, uint64_t *sums, hipStream_t st)
{
    const Tile *tiles = p.d_tiles + first;
    switch (esize) {
    case 1: k_generic<uint8_t, UNPACK, CSUM><<<count, kThreads, 0, st>>>(tiles, p.d_tensors, tensor_base, b, packed, sums); break;
    case 2: k_generic<uint16_t, UNPACK, CSUM><<<count, kThreads, 0, st>>>(tiles, p.d_tensors, tensor_base, b, packed, sums); break;
    case 4: k_generic<uint32_t, UNPACK, CSUM><<<count, kThreads, 0, st>>>(tiles, p.d_tensors, tensor_base, b, packed, sums); break;
    default: k_generic<uint64_t, UNPACK, CSUM><<<count, kThreads, 0, st>>>(tiles, p.d_tensors, tensor_base, b, packed, sums); break;
    }
}

int zero_sums(const Plan &p, uint64_t *sums, hipStream_t st)
{
    const uint32_t n = uint32_t(p.C);
    k_fill_zero<<<(n + kThreads - 1) / kThreads, kThreads, 0, st>>>(sums, n);
    HXT_HIP(hipGetLastError());
    return HXT_OK;
}

// The element size a launch of the per-element or transpose kernel is instantiated for is a
// property of the tensor, so such launches are issued per run of tiles with one element size.
template <bool UNPACK, bool CSUM>
int run_groups(const Plan &p, void *const *ptrs, uint8_t *packed, uint64_t *sums, hipStream_t st)
{
    for (const Group &g : p.groups) {
        BasePtrs b;
        std::memset(&b, 0, sizeof b);
        bool fast_ok = true;
        for (uint32_t i = 0; i < g.n_tensors; ++i) {
            const TensorPlan &tp = p.tensors[g.tensor_base + i];
            uint8_t *base = static_cast<uint8_t *>(ptrs[g.tensor_base + i]);
            b.p[i] = base;
            if (tp.bytes == 0) continue;
            if (!base) return HXT_EINVAL;
            if (reinterpret_cast<uintptr_t>(base) % tp.esize) return HXT_EALIGN;
            if ((tp.kind == K_CONTIG || tp.kind == K_ROWS) && tp.kind == g.kernel &&
                reinterpret_cast<uintptr_t>(base) % 16)
                fast_ok = false;
        }
        if (g.kernel == K_CONTIG && fast_ok) {
            launch_contig<UNPACK, CSUM>(p, g, b, packed, sums, st);
        } else if (g.kernel == K_ROWS && fast_ok) {
            launch_rows<UNPACK, CSUM>(p, g, b, packed, sums, st);
        } else {
            // split the group's tiles into runs of equal element size (host table, same order as the device one)
            uint32_t i = 0;
            while (i < g.count) {
                const int es = p.tensors[g.tensor_base + p.tiles[g.first + i].tensor].esize;
                uint32_t j = i + 1;
                while (j < g.count && p.tensors[g.tensor_base + p.tiles[g.first + j].tensor].esize == es) ++j;
                Group sub = g;
                sub.first = g.first + i;
                sub.count = j - i;
                if (g.kernel == K_TRANSPOSE)
                    launch_transpose<UNPACK, CSUM>(p, sub, es, b, packed, sums, st);
                else
                    launch_generic<UNPACK, CSUM>(p, sub.first, sub.count, g.tensor_base, es, b, packed, sums, st);
                i = j;
            }
        }
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
    if (!p.d_tiles) {
        g_last_hip = int(hipErrorNoDevice);
        return HXT_EHIP;
    }
    return HXT_OK;
}

int upload(Plan &p)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return HXT_OK;                      // no GPU: queries still work, data-plane calls report HXT_EHIP
    }
    p.device = dev;
    if (p.tiles.empty()) return HXT_OK;
    HXT_HIP(hipMalloc(reinterpret_cast<void **>(&p.d_tiles), p.tiles.size() * sizeof(Tile)));
    HXT_HIP(hipMemcpy(p.d_tiles, p.tiles.data(), p.tiles.size() * sizeof(Tile), hipMemcpyHostToDevice));
    if (!p.tdev.empty()) {
        HXT_HIP(hipMalloc(reinterpret_cast<void **>(&p.d_tensors), p.tdev.size() * sizeof(TensorDev)));
        HXT_HIP(hipMemcpy(p.d_tensors, p.tdev.data(), p.tdev.size() * sizeof(TensorDev), hipMemcpyHostToDevice));
    }
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

int stage(const hxt_plan_t *plan, int lane, const void *from, void *to, hipMemcpyKind kind, void *stream)
{
    if (!plan) return HXT_EINVAL;
    const Plan &p = plan->p;
    if (lane < -1 || lane >= p.k) return HXT_EINVAL;
    if (p.C == 0) return HXT_OK;
    if (!from || !to) return HXT_EINVAL;
    if (reinterpret_cast<uintptr_t>(from) % HXT_ALIGN || reinterpret_cast<uintptr_t>(to) % HXT_ALIGN) return HXT_EALIGN;
    uint64_t r[2][2];
    const int n = stage_ranges(p, lane, r);
    for (int i = 0; i < n; ++i)
        HXT_HIP(hipMemcpyAsync(static_cast<uint8_t *>(to) + r[i][0], static_cast<const uint8_t *>(from) + r[i][0],
                               r[i][1], kind, static_cast<hipStream_t>(stream)));
    return HXT_OK;
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
        if (rc == HXT_OK) rc = upload(pl->p);
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
    if (plan->p.d_tiles && hipFree(plan->p.d_tiles) != hipSuccess) rc = HXT_EHIP;
    if (plan->p.d_tensors && hipFree(plan->p.d_tensors) != hipSuccess) rc = HXT_EHIP;
    delete plan;
    return rc;
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
    if (!src) return HXT_EINVAL;
    const Plan &p = plan->p;
    hipStream_t st = static_cast<hipStream_t>(stream);
    void *const *ptrs = const_cast<void *const *>(src);
    // validate every pointer before anything is enqueued
    for (size_t i = 0; i < p.tensors.size(); ++i) {
        if (p.tensors[i].bytes == 0) continue;
        if (!ptrs[i]) return HXT_EINVAL;
        if (reinterpret_cast<uintptr_t>(ptrs[i]) % p.tensors[i].esize) return HXT_EALIGN;
    }
    if (sums) {
        rc = zero_sums(p, sums, st);
        if (rc != HXT_OK) return rc;
        return run_groups<false, true>(p, ptrs, static_cast<uint8_t *>(packed), sums, st);
    }
    return run_groups<false, false>(p, ptrs, static_cast<uint8_t *>(packed), nullptr, st);
}

int hxt_unpack(const hxt_plan_t *plan, const void *packed, void *const *dst, uint64_t *sums, void *stream)
{
    int rc = check_common(plan, packed);
    if (rc != HXT_OK || plan->p.C == 0) return rc;
    if (!dst) return HXT_EINVAL;
    const Plan &p = plan->p;
    if (!p.all_unpack_safe) return HXT_EOVERLAP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    for (size_t i = 0; i < p.tensors.size(); ++i) {
        if (p.tensors[i].bytes == 0) continue;
        if (!dst[i]) return HXT_EINVAL;
        if (reinterpret_cast<uintptr_t>(dst[i]) % p.tensors[i].esize) return HXT_EALIGN;
    }
    uint8_t *pk = const_cast<uint8_t *>(static_cast<const uint8_t *>(packed));
    if (sums) {
        rc = zero_sums(p, sums, st);
        if (rc != HXT_OK) return rc;
        return run_groups<true, true>(p, dst, pk, sums, st);
    }
    return run_groups<true, false>(p, dst, pk, nullptr, st);
}

int hxt_checksum(const hxt_plan_t *plan, const void *packed, uint64_t *sums, void *stream)
{
    int rc = check_common(plan, packed);
    if (rc != HXT_OK || plan->p.C == 0) return rc;
    if (!sums) return HXT_EINVAL;
    const Plan &p = plan->p;
    hipStream_t st = static_cast<hipStream_t>(stream);
    rc = zero_sums(p, sums, st);
    if (rc != HXT_OK) return rc;
    const Tile *tiles = p.d_tiles + p.csum_first;
    if (tuning().nt)
        k_checksum<kUnroll, true><<<p.csum_count, kThreads, 0, st>>>(tiles, static_cast<const uint8_t *>(packed), sums);
    else
        k_checksum<kUnroll, false><<<p.csum_count, kThreads, 0, st>>>(tiles, static_cast<const uint8_t *>(packed), sums);
    HXT_HIP(hipGetLastError());
    return HXT_OK;
}

int hxt_stage_d2h(const hxt_plan_t *plan, int lane, const void *packed_dev, void *host_pinned, void *stream)
{
    return stage(plan, lane, packed_dev, host_pinned, hipMemcpyDeviceToHost, stream);
}

int hxt_stage_h2d(const hxt_plan_t *plan, int lane, const void *host_pinned, void *packed_dev, void *stream)
{
    return stage(plan, lane, host_pinned, packed_dev, hipMemcpyHostToDevice, stream);
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

const char *hxt_version(void) { return "hxt 0.1 (gfx950)"; }

}  // extern "C"
