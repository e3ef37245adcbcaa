// HIP kernels (gfx950) of libhxt: device code only, included by hxt_device.hip.
//
// Data plane of the paper's Section 2.2 transfer: user buffer -> chunk buffer on
// the sender (pack), chunk buffer -> user buffer on the receiver (unpack), and a
// per-chunk integrity sum.  Every kernel is a pure byte mover: data is handled as
// unsigned integers so that any bit pattern survives unchanged.
//
// Work decomposition: the host planner cuts the message into tiles (one per
// workgroup, never crossing a tensor, and never a chunk except in
// k_transpose_span); a workgroup reads its 64-byte tile record with scalar
// loads and moves the bytes with 128-bit vector accesses where the view allows.
// Checksums are accumulated per thread in 64-bit integers, reduced across the
// 64-lane wavefront with shuffles, across the four waves through LDS, and added
// to the chunk's total with one 64-bit atomic per workgroup (k_transpose_span:
// one per chunk its tile touches); integer addition makes the result
// independent of the order of arrival.
#ifndef HXT_KERNELS_H
#define HXT_KERNELS_H

#include <hip/hip_runtime.h>

#include <cstdint>

#include "hxt_internal.h"

namespace hxt {

constexpr int kThreads = 256;
constexpr int kUnroll = 4;
constexpr uint32_t kTagMagic = 0x31545848u;     // 'H','X','T','1' in memory order

struct BasePtrs {
    uint8_t *p[kMaxGroupTensors];
};

struct ElemKinds {                     // per tensor of a launch group: 1 = 32-bit float, 0 = bf16
    uint8_t f32[kMaxGroupTensors];
};

// Accumulator slot of a checksum in flight.  Every operation of a plan (pack, unpack, the
// stand-alone passes, ...) owns its own set of slots, SumCtx::stride bytes apart (256 unless the
// plan has very many chunks) so that neighbouring slots' atomics land in different memory
// channels.  Always zero between kernels.
struct Acc {
    unsigned long long sum;
    uint32_t cnt;
    uint32_t pad;
};

struct SumCtx {
    uint64_t *sums;      // caller's array, one entry per chunk
    uint8_t *acc;        // plan-owned Acc slots: C * fan first-level slots, then C second-level slots
    uint32_t stride;     // bytes between slots
    uint32_t sum_bits;   // > 0: a chunk's total fits this many bits and the arrival count rides above it
    uint32_t fan;        // first-level slots per chunk (power of two); 1 = second level only
    uint32_t chunks;     // C
};

// ---- small device helpers ----------------------------------------------------

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <bool NT>
__device__ __forceinline__ u32x4 load16(const u32x4 *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}

template <bool NT>
__device__ __forceinline__ void store16(u32x4 *p, u32x4 v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

template <bool NT, typename E>
__device__ __forceinline__ E load_elem(const E *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}

template <bool NT, typename E>
__device__ __forceinline__ void store_elem(E *p, E v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// Vector v of a span of nvec (>= 1) vectors, zeros beyond its end.  The load itself is unconditional (the
// index is clamped into the span): the loads of an unrolled round are then all issued before the first
// of them is waited for, where guarded loads are waited for one by one.
template <bool NT>
__device__ __forceinline__ u32x4 load16_or_zero(const u32x4 *s, uint32_t v, uint32_t nvec)
{
    const u32x4 x = load16<NT>(s + min(v, nvec - 1));
    return v < nvec ? x : u32x4{0, 0, 0, 0};
}

__device__ __forceinline__ uint64_t words_sum(u32x4 v)
{
    return (uint64_t(v.x) + uint64_t(v.y)) + (uint64_t(v.z) + uint64_t(v.w));
}

// One arrival at an accumulator slot that expects `expected` of them: adds `value` and reports
// whether this was the last arrival, in which case `value` becomes the slot's total and the
// slot is zero again.  Only relaxed device-scope atomics touch a slot (no cache write-back).
//   sum_bits > 0: totals stay below 2^sum_bits (a chunk has at most B/4 words of 32 bits) and
//     the arrival count fits in the bits above, so one atomic adds and takes the ticket at once.
//   sum_bits == 0: sum and ticket are two words; the ticket is taken after the wave has seen
//     its own addition return, which orders the two.
__device__ __forceinline__ bool slot_arrive(Acc *a, unsigned long long &value, uint32_t expected, uint32_t sum_bits)
{
    if (expected == 1) return true;
    if (sum_bits) {
        const unsigned long long one = 1ull << sum_bits;
        const unsigned long long before = __hip_atomic_fetch_add(&a->sum, one + value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((before >> sum_bits) != expected - 1) return false;
        __hip_atomic_store(&a->sum, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        value = (before + value) & (one - 1);
        return true;
    }
    const unsigned long long before = __hip_atomic_fetch_add(&a->sum, value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("s_waitcnt vmcnt(0)" ::"v"(uint32_t(before)) : "memory");
    const uint32_t ticket = __hip_atomic_fetch_add(&a->cnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (ticket != expected - 1) return false;
    value = __hip_atomic_exchange(&a->sum, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(&a->cnt, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return true;
}

// Adds this workgroup's partial sum to its chunk.  A chunk made of many tiles spreads its
// arrivals over `fan` first-level slots (tile ordinal mod fan) so that they do not queue on
// one address; the last arrival of a first-level slot carries that slot's total to the chunk's
// second-level slot, and the last arrival there writes sums[chunk].
// One arrival, made by one thread: `s` is a finished partial sum for `chunk`, this being arrival number
// `ordinal` of the `expected` the chunk gets.
__device__ __forceinline__ void commit_total(unsigned long long s, uint32_t chunk, uint32_t ordinal, uint32_t expected,
                                             const SumCtx &cx)
{
    Acc *top = reinterpret_cast<Acc *>(cx.acc + (size_t(cx.chunks) * cx.fan + chunk) * cx.stride);
    bool last;
    if (cx.fan == 1 || expected < 2 * cx.fan) {
        last = slot_arrive(top, s, expected, cx.sum_bits);
    } else {
        const uint32_t sub = ordinal & (cx.fan - 1);
        const uint32_t share = expected / cx.fan + (sub < (expected & (cx.fan - 1)) ? 1u : 0u);
        Acc *first = reinterpret_cast<Acc *>(cx.acc + (size_t(chunk) * cx.fan + sub) * cx.stride);
        last = slot_arrive(first, s, share, cx.sum_bits) && slot_arrive(top, s, cx.fan, cx.sum_bits);
    }
    if (last) cx.sums[chunk] = s;
}

__device__ __forceinline__ void chunk_commit(uint64_t acc, uint32_t chunk, uint32_t ordinal, uint32_t expected,
                                             const SumCtx &cx)
{
    __shared__ uint64_t part[kThreads / 64];
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_down(acc, o, 64);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) part[wave] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long s = 0;
#pragma unroll
        for (int w = 0; w < kThreads / 64; ++w) s += part[w];
        commit_total(s, chunk, ordinal, expected, cx);
    }
}

// Copy `bytes` contiguous bytes between a user tensor and the packed buffer (pack: user ->
// packed, unpack: packed -> user) in 16-byte vectors, UNROLL independent loads in flight per
// thread before the first store; a last partial vector goes byte by byte.  NTU / NTP mark
// the user-side / packed-side accesses non-temporal; UA is the alignment of `user`.
// (The two blocks below are the user-side access helpers and the copy itself.)
// 16 bytes of a user tensor that is only UA-byte aligned (UA = 16, 4, 2 or 1): the vector is put
// together from / taken apart into naturally aligned pieces, so no access is misaligned and none
// touches a byte outside the 16.
template <int UA, bool NT>
__device__ __forceinline__ u32x4 load_user(const uint8_t *p)
{
    if constexpr (UA == 16) {
        return load16<NT>(reinterpret_cast<const u32x4 *>(p));
    } else if constexpr (UA == 4) {
        const uint32_t *q = reinterpret_cast<const uint32_t *>(p);
        return u32x4{q[0], q[1], q[2], q[3]};
    } else if constexpr (UA == 2) {
        const uint16_t *q = reinterpret_cast<const uint16_t *>(p);
        return u32x4{q[0] | uint32_t(q[1]) << 16, q[2] | uint32_t(q[3]) << 16, q[4] | uint32_t(q[5]) << 16,
                     q[6] | uint32_t(q[7]) << 16};
    } else {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            w[i] = p[4 * i] | uint32_t(p[4 * i + 1]) << 8 | uint32_t(p[4 * i + 2]) << 16 | uint32_t(p[4 * i + 3]) << 24;
        return u32x4{w[0], w[1], w[2], w[3]};
    }
}

template <int UA, bool NT>
__device__ __forceinline__ void store_user(uint8_t *p, u32x4 v)
{
    if constexpr (UA == 16) {
        store16<NT>(reinterpret_cast<u32x4 *>(p), v);
    } else if constexpr (UA == 4) {
        uint32_t *q = reinterpret_cast<uint32_t *>(p);
        q[0] = v.x, q[1] = v.y, q[2] = v.z, q[3] = v.w;
    } else if constexpr (UA == 2) {
        uint16_t *q = reinterpret_cast<uint16_t *>(p);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) q[2 * i] = uint16_t(w[i]), q[2 * i + 1] = uint16_t(w[i] >> 16);
    } else {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 16; ++i) p[i] = uint8_t(w[i >> 2] >> (8 * (i & 3)));
    }
}

template <bool UNPACK, bool CSUM, bool NTU, bool NTP, int UA = 16>
__device__ __forceinline__ uint64_t copy_span(uint8_t *user, uint8_t *pk, uint32_t bytes)
{
    const uint32_t nvec = bytes >> 4;
    constexpr uint32_t STEP = kThreads * kUnroll;
    const uint32_t full = nvec / STEP * STEP;            // uniform: blocks that need no bounds checks
    auto load = [&](uint32_t v) {
        if constexpr (UNPACK) return load16<NTP>(reinterpret_cast<const u32x4 *>(pk) + v);
        else return load_user<UA, NTU>(user + (size_t(v) << 4));
    };
    auto store = [&](uint32_t v, u32x4 r) {
        if constexpr (UNPACK) store_user<UA, NTU>(user + (size_t(v) << 4), r);
        else store16<NTP>(reinterpret_cast<u32x4 *>(pk) + v, r);
    };
    uint64_t acc = 0;
    for (uint32_t v = threadIdx.x; v < full; v += STEP) {
        u32x4 r[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) r[u] = load(v + u * kThreads);
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            store(v + u * kThreads, r[u]);
            if constexpr (CSUM) acc += words_sum(r[u]);
        }
    }
    for (uint32_t v = full + threadIdx.x; v < nvec; v += kThreads) {
        const u32x4 r = load(v);
        store(v, r);
        if constexpr (CSUM) acc += words_sum(r);
    }
    const uint32_t tail = bytes & 15;                    // only at the very end of a tensor
    if (threadIdx.x < tail) {
        const uint32_t i = (nvec << 4) + threadIdx.x;
        const uint8_t b = (UNPACK ? pk : user)[i];
        (UNPACK ? user : pk)[i] = b;
        if constexpr (CSUM) acc += uint64_t(b) << (8 * (i & 3));
    }
    return acc;
}

// ---- receive and accumulate -----------------------------------------------------
// new = round(old + arriving) per element.  bf16: both operands widened exactly to binary32,
// added in binary32, the sum rounded to bf16 to nearest with ties to even.  f32: binary32
// addition.  Every NaN result becomes the canonical quiet NaN, so that the outcome does not
// depend on NaN payload propagation.
__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f)
{
    const uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0u;
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

__device__ __forceinline__ uint32_t add_bf16x2(uint32_t old, uint32_t in)
{
    const float lo = __uint_as_float(old << 16) + __uint_as_float(in << 16);
    const float hi = __uint_as_float(old & 0xFFFF0000u) + __uint_as_float(in & 0xFFFF0000u);
    return f32_to_bf16_rne(lo) | (f32_to_bf16_rne(hi) << 16);
}

__device__ __forceinline__ uint32_t add_f32(uint32_t old, uint32_t in)
{
    const uint32_t u = __float_as_uint(__uint_as_float(old) + __uint_as_float(in));
    return (u & 0x7FFFFFFFu) > 0x7F800000u ? 0x7FC00000u : u;
}

template <bool F32>
__device__ __forceinline__ u32x4 add_vec(u32x4 old, u32x4 in)
{
    if constexpr (F32) return u32x4{add_f32(old.x, in.x), add_f32(old.y, in.y), add_f32(old.z, in.z), add_f32(old.w, in.w)};
    else return u32x4{add_bf16x2(old.x, in.x), add_bf16x2(old.y, in.y), add_bf16x2(old.z, in.z), add_bf16x2(old.w, in.w)};
}

// Adds `bytes` arriving contiguous bytes at pk to the tensor bytes at user (both 16-byte aligned
// except for a last partial vector, which goes element by element).  Returns the checksum
// contribution of the packed bytes read.
template <bool F32, bool CSUM, bool NTU, bool NTP, int UA = 16>
__device__ __forceinline__ uint64_t accumulate_span(uint8_t *user, const uint8_t *pk, uint32_t bytes)
{
    const u32x4 *in = reinterpret_cast<const u32x4 *>(pk);
    const uint32_t nvec = bytes >> 4;
    constexpr int U = 2;                                   // two vectors of each operand in flight per thread
    constexpr uint32_t STEP = kThreads * U;
    const uint32_t full = nvec / STEP * STEP;
    uint64_t acc = 0;
    for (uint32_t v = threadIdx.x; v < full; v += STEP) {
        u32x4 a[U], b[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            a[u] = load16<NTP>(in + v + u * kThreads);
            b[u] = load_user<UA, NTU>(user + (size_t(v + u * kThreads) << 4));
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            store_user<UA, NTU>(user + (size_t(v + u * kThreads) << 4), add_vec<F32>(b[u], a[u]));
            if constexpr (CSUM) acc += words_sum(a[u]);
        }
    }
    for (uint32_t v = full + threadIdx.x; v < nvec; v += kThreads) {
        const u32x4 a = load16<NTP>(in + v);
        uint8_t *at = user + (size_t(v) << 4);
        store_user<UA, NTU>(at, add_vec<F32>(load_user<UA, NTU>(at), a));
        if constexpr (CSUM) acc += words_sum(a);
    }
    constexpr uint32_t ES = F32 ? 4 : 2;
    const uint32_t tail = (bytes & 15) / ES;               // whole elements in the last partial vector
    if (threadIdx.x < tail) {
        const uint32_t off = (nvec << 4) + threadIdx.x * ES;
        if constexpr (F32) {
            const uint32_t a = *reinterpret_cast<const uint32_t *>(pk + off);
            uint32_t *d = reinterpret_cast<uint32_t *>(user + off);
            *d = add_f32(*d, a);
            if constexpr (CSUM) acc += a;
        } else {
            const uint32_t a = *reinterpret_cast<const uint16_t *>(pk + off);
            uint16_t *d = reinterpret_cast<uint16_t *>(user + off);
            *d = uint16_t(add_bf16x2(*d, a));
            if constexpr (CSUM) acc += uint64_t(a) << (8 * (off & 3));
        }
    }
    return acc;
}

// Pad bytes (fewer than 256): pack writes zeros, unpack only reads them for the sum.
// `phase` is the position of pk[0] within its 32-bit word.
template <bool UNPACK, bool CSUM>
__device__ __forceinline__ uint64_t pad_span(uint8_t *pk, uint32_t bytes, uint32_t phase)
{
    uint64_t acc = 0;
    for (uint32_t i = threadIdx.x; i < bytes; i += kThreads) {
        if constexpr (!UNPACK) pk[i] = 0;
        if constexpr (UNPACK && CSUM) acc += uint64_t(pk[i]) << (8 * ((phase + i) & 3));
    }
    return acc;
}

// ---- uniform copy: messages that are one contiguous tensor each -------------------
// No table: tile -> (chunk, lane, slot, offsets) in closed form from the kernel arguments.
// One launch can serve several such messages (the forward activation and the backward
// gradient that cross a stage boundary at the same point of the schedule): workgroups
// [first_tile, first_tile + ntiles) belong to message i.
constexpr int kMaxBatch = 4;

struct UniformItem {
    ChunkGeom g;
    uint8_t *user;
    uint8_t *packed;
    SumCtx cx;
    uint32_t first_tile;
    uint32_t unpack;       // direction of this item; only read by the mixed-direction instantiation
};

enum Direction { DIR_PACK = 0, DIR_UNPACK = 1, DIR_MIXED = 2 };

struct UniformArgs {
    UniformItem it[kMaxBatch];
    uint32_t n;
};

template <bool UNPACK, bool CSUM, bool NTU, bool NTP>
__device__ __forceinline__ void uniform_tile(const UniformItem &it, uint32_t tile)
{
    const ChunkGeom &g = it.g;
    const TileSpan t = locate_tile(g, tile);
    const uint64_t left = g.N > t.stream_off ? g.N - t.stream_off : 0;     // tensor bytes from here on
    const uint32_t data = left < t.len ? uint32_t(left) : t.len;
    uint8_t *pk = it.packed + t.packed_off;
    uint64_t acc = copy_span<UNPACK, CSUM, NTU, NTP>(it.user + t.stream_off, pk, data);
    if (data < t.len) acc += pad_span<UNPACK, CSUM>(pk + data, t.len - data, data);
    if constexpr (CSUM) chunk_commit(acc, t.chunk, t.ordinal, t.expected, it.cx);
}

// DIR: all items pack, all unpack, or each item says which (a micro-batch stream overlaps the
// unpack of one message with the pack of the next inside one launch).
template <int DIR, bool CSUM, bool NTU, bool NTP>
__global__ __launch_bounds__(kThreads) void k_uniform(UniformArgs a)
{
    uint32_t m = 0;
#pragma unroll
    for (uint32_t i = 1; i < kMaxBatch; ++i)
        if (i < a.n && blockIdx.x >= a.it[i].first_tile) m = i;
    const UniformItem &it = a.it[m];
    const uint32_t tile = blockIdx.x - it.first_tile;
    if constexpr (DIR == DIR_MIXED) {
        if (it.unpack) uniform_tile<true, CSUM, NTU, NTP>(it, tile);
        else uniform_tile<false, CSUM, NTU, NTP>(it, tile);
    } else {
        uniform_tile<DIR == DIR_UNPACK, CSUM, NTU, NTP>(it, tile);
    }
}

// ---- contiguous tensors of a multi-tensor message: table driven ---------------------
template <bool UNPACK, bool CSUM, bool NTU, bool NTP>
__global__ __launch_bounds__(kThreads) void k_contig(const Tile *__restrict__ tiles,
                                                     const uint32_t *__restrict__ chunk_tiles, BasePtrs bases,
                                                     uint8_t *__restrict__ packed, SumCtx cx)
{
    const Tile t = tiles[blockIdx.x];
    uint64_t acc;
    if (t.kind == K_ZERO)
        acc = pad_span<UNPACK, CSUM>(packed + t.packed_off, t.n0, uint32_t(t.packed_off));
    else
        acc = copy_span<UNPACK, CSUM, NTU, NTP>(bases.p[t.tensor] + t.src_off, packed + t.packed_off, t.n0);
    if constexpr (CSUM) chunk_commit(acc, t.chunk, t.ordinal, chunk_tiles[t.chunk], cx);
}

// ---- contiguous tensors whose base pointer is only element aligned -------------------
// The same copies with the user side accessed in pieces of its actual alignment (4, 2 or 1 bytes;
// the packed side stays 16 bytes wide).  Separate kernels, so that the aligned ones keep their
// register budget.
template <bool UNPACK, bool CSUM>
__device__ __forceinline__ uint64_t copy_span_any(uint8_t *user, uint8_t *pk, uint32_t bytes)
{
    const uint32_t mis = uint32_t(reinterpret_cast<uintptr_t>(user)) & 15u;          // the same for the whole workgroup
    if (mis == 0) return copy_span<UNPACK, CSUM, false, false, 16>(user, pk, bytes);
    if ((mis & 3u) == 0) return copy_span<UNPACK, CSUM, false, false, 4>(user, pk, bytes);
    if ((mis & 1u) == 0) return copy_span<UNPACK, CSUM, false, false, 2>(user, pk, bytes);
    return copy_span<UNPACK, CSUM, false, false, 1>(user, pk, bytes);
}

template <bool UNPACK, bool CSUM>
__global__ __launch_bounds__(kThreads) void k_uniform_any(UniformArgs a)
{
    const UniformItem &it = a.it[0];
    const ChunkGeom &g = it.g;
    const TileSpan t = locate_tile(g, blockIdx.x);
    const uint64_t left = g.N > t.stream_off ? g.N - t.stream_off : 0;
    const uint32_t data = left < t.len ? uint32_t(left) : t.len;
    uint8_t *pk = it.packed + t.packed_off;
    uint64_t acc = copy_span_any<UNPACK, CSUM>(it.user + t.stream_off, pk, data);
    if (data < t.len) acc += pad_span<UNPACK, CSUM>(pk + data, t.len - data, data);
    if constexpr (CSUM) chunk_commit(acc, t.chunk, t.ordinal, t.expected, it.cx);
}

template <bool UNPACK, bool CSUM>
__global__ __launch_bounds__(kThreads) void k_contig_any(const Tile *__restrict__ tiles,
                                                         const uint32_t *__restrict__ chunk_tiles, BasePtrs bases,
                                                         uint8_t *__restrict__ packed, SumCtx cx)
{
    const Tile t = tiles[blockIdx.x];
    uint64_t acc;
    if (t.kind == K_ZERO)
        acc = pad_span<UNPACK, CSUM>(packed + t.packed_off, t.n0, uint32_t(t.packed_off));
    else
        acc = copy_span_any<UNPACK, CSUM>(bases.p[t.tensor] + t.src_off, packed + t.packed_off, t.n0);
    if constexpr (CSUM) chunk_commit(acc, t.chunk, t.ordinal, chunk_tiles[t.chunk], cx);
}

// ---- receive and accumulate: the uniform and the table-driven contiguous kernels -----
template <bool CSUM, bool NTU, bool NTP>
__global__ __launch_bounds__(kThreads) void k_uniform_accumulate(UniformArgs a)
{
    uint32_t m = 0;                                    // up to kMaxBatch messages per launch, as in k_uniform
#pragma unroll
    for (uint32_t i = 1; i < kMaxBatch; ++i)
        if (i < a.n && blockIdx.x >= a.it[i].first_tile) m = i;
    const UniformItem &it = a.it[m];
    const ChunkGeom &g = it.g;
    const TileSpan t = locate_tile(g, blockIdx.x - it.first_tile);
    const uint64_t left = g.N > t.stream_off ? g.N - t.stream_off : 0;
    const uint32_t data = left < t.len ? uint32_t(left) : t.len;
    uint8_t *pk = it.packed + t.packed_off;
    uint64_t acc = it.unpack ? accumulate_span<true, CSUM, NTU, NTP>(it.user + t.stream_off, pk, data)
                             : accumulate_span<false, CSUM, NTU, NTP>(it.user + t.stream_off, pk, data);
    if (data < t.len) acc += pad_span<true, CSUM>(pk + data, t.len - data, data);
    if constexpr (CSUM) chunk_commit(acc, t.chunk, t.ordinal, t.expected, it.cx);
}

// The same for destinations whose base is only element aligned.
template <bool F32, bool CSUM>
__device__ __forceinline__ uint64_t accumulate_span_any(uint8_t *user, const uint8_t *pk, uint32_t bytes)
{
    const uint32_t mis = uint32_t(reinterpret_cast<uintptr_t>(user)) & 15u;
    if (mis == 0) return accumulate_span<F32, CSUM, false, false, 16>(user, pk, bytes);
    if ((mis & 3u) == 0) return accumulate_span<F32, CSUM, false, false, 4>(user, pk, bytes);
    return accumulate_span<F32, CSUM, false, false, 2>(user, pk, bytes);      // bf16 on an odd element
}

template <bool CSUM>
__global__ __launch_bounds__(kThreads) void k_uniform_accumulate_any(UniformArgs a)
{
    const UniformItem &it = a.it[0];
    const ChunkGeom &g = it.g;
    const TileSpan t = locate_tile(g, blockIdx.x);
    const uint64_t left = g.N > t.stream_off ? g.N - t.stream_off : 0;
    const uint32_t data = left < t.len ? uint32_t(left) : t.len;
    uint8_t *pk = it.packed + t.packed_off;
    uint64_t acc = it.unpack ? accumulate_span_any<true, CSUM>(it.user + t.stream_off, pk, data)
                             : accumulate_span_any<false, CSUM>(it.user + t.stream_off, pk, data);
    if (data < t.len) acc += pad_span<true, CSUM>(pk + data, t.len - data, data);
    if constexpr (CSUM) chunk_commit(acc, t.chunk, t.ordinal, t.expected, it.cx);
}

template <bool CSUM>
__global__ __launch_bounds__(kThreads) void k_contig_accumulate_any(const Tile *__restrict__ tiles,
                                                                    const uint32_t *__restrict__ chunk_tiles,
                                                                    BasePtrs bases, ElemKinds kinds,
                                                                    uint8_t *__restrict__ packed, SumCtx cx)
{
    const Tile t = tiles[blockIdx.x];
    uint64_t acc;
    if (t.kind == K_ZERO)
        acc = pad_span<true, CSUM>(packed + t.packed_off, t.n0, uint32_t(t.packed_off));
    else if (kinds.f32[t.tensor])
        acc = accumulate_span_any<true, CSUM>(bases.p[t.tensor] + t.src_off, packed + t.packed_off, t.n0);
    else
        acc = accumulate_span_any<false, CSUM>(bases.p[t.tensor] + t.src_off, packed + t.packed_off, t.n0);
    if constexpr (CSUM) chunk_commit(acc, t.chunk, t.ordinal, chunk_tiles[t.chunk], cx);
}

template <bool CSUM, bool NTU, bool NTP>
__global__ __launch_bounds__(kThreads) void k_contig_accumulate(const Tile *__restrict__ tiles,
                                                                const uint32_t *__restrict__ chunk_tiles,
                                                                BasePtrs bases, ElemKinds kinds,
                                                                uint8_t *__restrict__ packed, SumCtx cx)
{
    const Tile t = tiles[blockIdx.x];
    uint64_t acc;
    if (t.kind == K_ZERO)
        acc = pad_span<true, CSUM>(packed + t.packed_off, t.n0, uint32_t(t.packed_off));
    else if (kinds.f32[t.tensor])
        acc = accumulate_span<true, CSUM, NTU, NTP>(bases.p[t.tensor] + t.src_off, packed + t.packed_off, t.n0);
    else
        acc = accumulate_span<false, CSUM, NTU, NTP>(bases.p[t.tensor] + t.src_off, packed + t.packed_off, t.n0);
    if constexpr (CSUM) chunk_commit(acc, t.chunk, t.ordinal, chunk_tiles[t.chunk], cx);
}

// ---- rows: innermost dimension contiguous, outer dimensions strided -------------
// A 16-byte vector never straddles a run (run length and strides are multiples of 16).
// Logical byte -> (row, column) and row -> outer indices use multiply-shift division.
template <bool UNPACK, bool CSUM, bool NTU, bool NTP, int UA>
__device__ __forceinline__ uint64_t rows_tile(const Tile &t, const TensorDev &td, uint8_t *user, uint8_t *pk)
{
    const uint32_t row_bytes = td.row_bytes;
    const uint64_t row0 = t.src_off / row_bytes;                    // uniform
    const uint32_t col0 = uint32_t(t.src_off - row0 * row_bytes);
    const int outer = td.ndim - 1;
    const uint32_t nvec = t.n0 >> 4;
    uint64_t acc = 0;
    for (uint32_t v0 = threadIdx.x; v0 < nvec; v0 += kThreads * kUnroll) {
        u32x4 r[kUnroll];
        uint64_t off[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
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
            if (v < nvec) {
                if constexpr (UNPACK) r[u] = load16<NTP>(reinterpret_cast<const u32x4 *>(pk + (uint64_t(v) << 4)));
                else r[u] = load_user<UA, NTU>(user + o);
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const uint32_t v = v0 + u * kThreads;
            if (v < nvec) {
                if constexpr (UNPACK) store_user<UA, NTU>(user + off[u], r[u]);
                else store16<NTP>(reinterpret_cast<u32x4 *>(pk + (uint64_t(v) << 4)), r[u]);
                if constexpr (CSUM) acc += words_sum(r[u]);
            }
        }
    }
    return acc;
}

template <bool UNPACK, bool CSUM, bool NTU, bool NTP>
__global__ __launch_bounds__(kThreads) void k_rows(const Tile *__restrict__ tiles,
                                                   const uint32_t *__restrict__ chunk_tiles,
                                                   const TensorDev *__restrict__ tensors, uint32_t tensor_base,
                                                   BasePtrs bases, uint8_t *__restrict__ packed, SumCtx cx)
{
    const Tile t = tiles[blockIdx.x];
    const uint64_t acc = rows_tile<UNPACK, CSUM, NTU, NTP, 16>(t, tensors[tensor_base + t.tensor], bases.p[t.tensor],
                                                               packed + t.packed_off);
    if constexpr (CSUM) chunk_commit(acc, t.chunk, t.ordinal, chunk_tiles[t.chunk], cx);
}

// The same gather when a base pointer is only element aligned (all strides are multiples of 16 bytes, so
// every vector of a tensor is off by the same amount): narrower accesses on the tensor side.
template <bool UNPACK, bool CSUM>
__global__ __launch_bounds__(kThreads) void k_rows_any(const Tile *__restrict__ tiles,
                                                       const uint32_t *__restrict__ chunk_tiles,
                                                       const TensorDev *__restrict__ tensors, uint32_t tensor_base,
                                                       BasePtrs bases, uint8_t *__restrict__ packed, SumCtx cx)
{
    const Tile t = tiles[blockIdx.x];
    const TensorDev &td = tensors[tensor_base + t.tensor];
    uint8_t *user = bases.p[t.tensor], *pk = packed + t.packed_off;
    const uint32_t mis = uint32_t(reinterpret_cast<uintptr_t>(user)) & 15u;
    uint64_t acc;
    if (mis == 0) acc = rows_tile<UNPACK, CSUM, false, false, 16>(t, td, user, pk);
    else if ((mis & 3u) == 0) acc = rows_tile<UNPACK, CSUM, false, false, 4>(t, td, user, pk);
    else if ((mis & 1u) == 0) acc = rows_tile<UNPACK, CSUM, false, false, 2>(t, td, user, pk);
    else acc = rows_tile<UNPACK, CSUM, false, false, 1>(t, td, user, pk);
    if constexpr (CSUM) chunk_commit(acc, t.chunk, t.ordinal, chunk_tiles[t.chunk], cx);
}

// ---- rows whose length or pitch is not a multiple of 16 bytes ----------------------
// Still a gather of contiguous runs (of 16 bytes or more), but a 16-byte vector of the packed stream may end
// one run and begin the next, and the tensor side is only G-byte aligned (G = 8, 4, 2 or 1).
// Work is dealt in pieces of G bytes, consecutive lanes taking consecutive pieces of the tile: a wave's access
// is then contiguous on the packed side and contiguous within each run on the tensor side (64 lanes x 4 bytes
// = 256 bytes per instruction), whatever the run length; each piece finds its run with one multiply-shift
// division and the run's storage offset from the outer indices.
template <int G> struct PieceOf;
template <> struct PieceOf<8> { using type = uint64_t; };
template <> struct PieceOf<4> { using type = uint32_t; };
template <> struct PieceOf<2> { using type = uint16_t; };
template <> struct PieceOf<1> { using type = uint8_t; };

// TWO_D: the view has two dims (the usual padded-pitch matrix) and needs no index decomposition: run
// row0 + dr starts (row0 + dr) * pitch into the storage, so byte x of the tile's first run sits at
// x + dr * (pitch - run length) from that run's start.  Otherwise the run's storage offset comes from
// its outer indices, divided out with the dims held in registers (the loop stores through byte
// pointers, which may alias the descriptor, so anything read through it inside the loop would be
// read again for every piece).  With pieces of 1 or 2 bytes the loads of a round are unconditional
// (the piece number is clamped into the tile): guarded, the compiler waits for each load before it
// goes on to the next guard, and 16 loads one after the other cost 1.8-2.4 times the time.  With pieces
// of 4 or 8 bytes the guarded loads are issued without such waits, interleaved with the address
// arithmetic, and that order measures 10 % faster than eight loads in one burst.
template <bool UNPACK, bool CSUM, bool NTP, int G, bool TWO_D>
__device__ __forceinline__ uint64_t rows_split_tile(const Tile &t, const TensorDev &td, uint8_t *user, uint8_t *pk)
{
    using P = typename PieceOf<G>::type;
    const uint32_t row_bytes = td.row_bytes;
    const FastDiv row_div = td.row_div;
    const uint64_t row0 = t.src_off / row_bytes;                    // uniform
    const uint32_t col0 = uint32_t(t.src_off - row0 * row_bytes);
    const uint32_t npiece = t.n0 / G;
    constexpr int U = G == 8 ? 8 : 16;                              // pieces in flight per thread: a 16 KiB tile in one go
    constexpr int D = TWO_D ? 1 : HXT_MAX_DIMS - 1;                 // dims outside the run
    const int outer = TWO_D ? 1 : td.ndim - 1;
    uint32_t shape[D], mul[D], shift[D];
    uint64_t stride[D];
#pragma unroll
    for (int d = 0; d < D; ++d) {
        shape[d] = 1, mul[d] = 0, shift[d] = 0, stride[d] = 0;
        if (d < outer) {
            shape[d] = uint32_t(td.shape[d]);
            mul[d] = td.dim_div[d].mul;
            shift[d] = td.dim_div[d].shift;
            stride[d] = uint64_t(td.stride_b[d]);
        }
    }
    uint8_t *const first_run = user + row0 * stride[0];             // uniform
    const int64_t slack = int64_t(stride[0]) - int64_t(row_bytes);
    auto user_piece = [&](uint32_t i) {                             // piece i of the tile -> its place in storage
        const uint32_t x = col0 + i * G;
        const uint32_t dr = fast_div(x, row_div);
        if constexpr (TWO_D) {
            return reinterpret_cast<P *>(first_run + (int64_t(x) + int64_t(dr) * slack));
        } else {
            uint32_t row = uint32_t(row0) + dr;
            uint64_t o = 0;
#pragma unroll
            for (int d = D - 1; d > 0; --d) {
                if (d < outer) {
                    const uint32_t q = fast_div(row, FastDiv{mul[d], shift[d]});
                    o += uint64_t(row - q * shape[d]) * stride[d];
                    row = q;
                }
            }
            return reinterpret_cast<P *>(user + o + uint64_t(row) * stride[0] + (x - dr * row_bytes));
        }
    };
    P *pieces = reinterpret_cast<P *>(pk);
    uint64_t acc = 0;
    const uint32_t last = npiece - 1;
    for (uint32_t i0 = threadIdx.x; i0 < npiece; i0 += kThreads * U) {
        P r[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if constexpr (G >= 4) {
                const uint32_t i = i0 + u * kThreads;
                r[u] = 0;
                if (i < npiece) {
                    if constexpr (UNPACK) r[u] = load_elem<NTP>(pieces + i);
                    else r[u] = __builtin_nontemporal_load(user_piece(i));
                }
            } else {
                const uint32_t i = min(i0 + u * kThreads, last);
                if constexpr (UNPACK) r[u] = load_elem<NTP>(pieces + i);
                else r[u] = __builtin_nontemporal_load(user_piece(i));
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t i = i0 + u * kThreads;
            if (i < npiece) {
                if constexpr (UNPACK) __builtin_nontemporal_store(r[u], user_piece(i));
                else store_elem<NTP>(pieces + i, r[u]);
                if constexpr (CSUM && G == 8) acc += (uint64_t(r[u]) & 0xFFFFFFFFull) + (uint64_t(r[u]) >> 32);
                if constexpr (CSUM && G < 8) acc += uint64_t(r[u]) << (8 * ((i * G) & 3));
            }
        }
    }
    return acc;
}

template <bool UNPACK, bool CSUM, bool NTP>
__global__ __launch_bounds__(kThreads) void k_rows_split(const Tile *__restrict__ tiles,
                                                         const uint32_t *__restrict__ chunk_tiles,
                                                         const TensorDev *__restrict__ tensors, uint32_t tensor_base,
                                                         BasePtrs bases, uint8_t *__restrict__ packed, SumCtx cx)
{
    const Tile t = tiles[blockIdx.x];
    const TensorDev &td = tensors[tensor_base + t.tensor];
    uint8_t *user = bases.p[t.tensor], *pk = packed + t.packed_off;
    // widest piece that is naturally aligned everywhere: low bits of the base address, the run length and the pitches
    const uint32_t low = (uint32_t(reinterpret_cast<uintptr_t>(user)) | td.low_or) & 15u;
    auto run = [&]<int G>() {
        return td.ndim == 2 ? rows_split_tile<UNPACK, CSUM, NTP, G, true>(t, td, user, pk)
                            : rows_split_tile<UNPACK, CSUM, NTP, G, false>(t, td, user, pk);
    };
    uint64_t acc;
    if ((low & 7u) == 0) acc = run.template operator()<8>();
    else if ((low & 3u) == 0) acc = run.template operator()<4>();
    else if ((low & 1u) == 0) acc = run.template operator()<2>();
    else acc = run.template operator()<1>();
    if constexpr (CSUM) chunk_commit(acc, t.chunk, t.ordinal, chunk_tiles[t.chunk], cx);
}

// ---- transpose: logical inner dimension strided, the one before it contiguous ----
// A tile is ni x nj elements (at most 128 x 128 for 1- and 2-byte elements, 64 x 64 otherwise).  Storage is read/written along i, the packed
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

// Vector path of the transpose: src has R rows of Cc contiguous elements, dst gets Cc rows of R
// contiguous elements, dst[c][r] = src[r][c]; R and Cc are multiples of V = 16 / sizeof(E) and
// every row start is 16-byte aligned.  16-byte global loads along src rows land in LDS rows of
// T elements whose 16-byte slots are XOR-swizzled with the row group, so that the V element
// reads that assemble one dst vector (same column, V consecutive rows) and the other lanes'
// reads of the same instruction fall into distinct banks; then 16-byte global stores along dst
// rows.  The sum is taken on whichever side is the packed buffer.
// FULL: the tile is T x T, so every index computation folds to shifts and masks and each thread moves exactly
// T * T / (V * kThreads) vectors per phase, all of whose global loads are issued before the first LDS store
// (measured with counters: with run-time extents the kernel was bound by its integer divisions, not by memory).
// Where the rows of a tile lie on the packed side, and where their sums go.
// PitchRows: a tile inside one chunk, rows a fixed pitch apart, one sum for the tile.
struct PitchRows {
    uint8_t *base;
    uint64_t pitch;
    __device__ __forceinline__ uint8_t *at(uint32_t row, uint32_t byte) const { return base + row * pitch + byte; }
    __device__ __forceinline__ void count(uint32_t, uint32_t, uint64_t s, uint64_t &acc) const { acc += s; }
};
// SpanRows: every row placed on its own (k_transpose_span keeps the placement in LDS): bytes below first_b[row]
// lie p0[row] into the packed buffer, the rest p1[row]; a vector's sum goes to the partial sum of its chunk.
struct SpanRows {
    uint8_t *packed;
    const uint64_t *p0, *p1;
    const uint32_t *first_b, *entry;
    unsigned long long *part;
    __device__ __forceinline__ uint8_t *at(uint32_t row, uint32_t byte) const
    {
        return packed + (byte < first_b[row] ? p0[row] : p1[row]) + byte;
    }
    __device__ __forceinline__ void count(uint32_t row, uint32_t byte, uint64_t s, uint64_t &) const
    {
        __hip_atomic_fetch_add(&part[entry[row] + (byte < first_b[row] ? 0u : 1u)], (unsigned long long)s, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_WORKGROUP);
    }
};

// user / user_pitch: the tensor side (rows of the tile as the tensor stores them); pk: the packed side.
// SRC_IS_PACKED: unpack (packed rows are the source), else pack.
template <typename E, bool SRC_IS_PACKED, bool CSUM, bool NTP, int UA, bool FULL, class PK>
__device__ __forceinline__ uint64_t transpose_vec(uint8_t *user, uint64_t user_pitch, uint32_t R_in, uint32_t Cc_in,
                                                  const PK &pk, uint8_t *lds)
{
    constexpr uint32_t T = transpose_tile(sizeof(E)), V = 16 / sizeof(E), ROWB = T * sizeof(E), NV = T / V;
    const uint32_t R = FULL ? T : R_in, Cc = FULL ? T : Cc_in;
    uint64_t acc = 0;
    const uint32_t nvs = Cc / V;                           // vectors per src row
    auto load_src = [&](uint32_t v, uint32_t &slot) {
        const uint32_t r = v / nvs, cv = v - r * nvs;
        slot = r * ROWB + ((cv ^ ((r / V) % NV)) * 16);
        // the user tensor is streamed once (non-temporal) and may be only UA-byte aligned; the packed side as the plan says
        if constexpr (SRC_IS_PACKED) return load16<NTP>(reinterpret_cast<const u32x4 *>(pk.at(r, cv * 16)));
        else return load_user<UA, true>(user + r * user_pitch + cv * 16);
    };
    auto count_src = [&](uint32_t v, const u32x4 &x) {     // after the loads, so that none of them waits for a sum
        if constexpr (CSUM && SRC_IS_PACKED) {
            const uint32_t r = v / nvs, cv = v - r * nvs;
            pk.count(r, cv * 16, words_sum(x), acc);
        }
    };
    if constexpr (FULL) {
        constexpr uint32_t PER = T * T / (V * kThreads);   // 8 vectors per thread (4 for 1-byte elements)
        u32x4 x[PER];
        uint32_t slot[PER];
#pragma unroll
        for (uint32_t u = 0; u < PER; ++u) x[u] = load_src(threadIdx.x + u * kThreads, slot[u]);
#pragma unroll
        for (uint32_t u = 0; u < PER; ++u) {
            count_src(threadIdx.x + u * kThreads, x[u]);
            *reinterpret_cast<u32x4 *>(lds + slot[u]) = x[u];
        }
    } else {
        for (uint32_t v = threadIdx.x; v < R * nvs; v += kThreads) {
            uint32_t slot;
            const u32x4 x = load_src(v, slot);
            count_src(v, x);
            *reinterpret_cast<u32x4 *>(lds + slot) = x;
        }
    }
    __syncthreads();
    // dst vectors are handed out with 8 consecutive vectors of one dst row (128 contiguous bytes) fastest,
    // then the dst row: a half-wave then reads 8 row groups x 4 columns from LDS, which the swizzle spreads
    // over all 32 banks (16 row groups of one column pair would hit each bank twice).
    const uint32_t nvd = R / V;                            // vectors per dst row
    const uint32_t full8 = nvd >> 3, rem = nvd & 7, main = Cc * 8 * full8;
    auto move_dst = [&](uint32_t v) {
        uint32_t c, dv;
        if (FULL || v < main) {                            // a full tile's dst rows are whole groups of 8 vectors
            const uint32_t b = v / (Cc * 8), w = v - b * (Cc * 8);
            c = w >> 3;
            dv = b * 8 + (w & 7);
        } else if constexpr (!FULL) {
            const uint32_t w = v - main;
            c = w / rem;
            dv = full8 * 8 + (w - c * rem);
        }
        union {
            E e[V];
            u32x4 x;
        } o;
#pragma unroll
        for (uint32_t q = 0; q < V; ++q) {
            const uint32_t r = dv * V + q;
            o.e[q] = *reinterpret_cast<const E *>(lds + r * ROWB + (((c / V) ^ ((r / V) % NV)) * 16) + (c % V) * sizeof(E));
        }
        if constexpr (CSUM && !SRC_IS_PACKED) pk.count(c, dv * 16, words_sum(o.x), acc);
        if constexpr (SRC_IS_PACKED) store_user<UA, true>(user + c * user_pitch + dv * 16, o.x);
        else store16<NTP>(reinterpret_cast<u32x4 *>(pk.at(c, dv * 16)), o.x);
    };
    if constexpr (FULL) {
        static_assert(NV % 8 == 0, "a full tile's dst rows must be whole groups of 8 vectors");
        constexpr uint32_t PER = T * T / (V * kThreads);
#pragma unroll
        for (uint32_t u = 0; u < PER; ++u) move_dst(threadIdx.x + u * kThreads);
    } else {
        for (uint32_t v = threadIdx.x; v < Cc * nvd; v += kThreads) move_dst(v);
    }
    return acc;
}

template <typename E, bool UNPACK, bool CSUM, bool NTP>
__global__ __launch_bounds__(kThreads) void k_transpose(const Tile *__restrict__ tiles,
                                                        const uint32_t *__restrict__ chunk_tiles, BasePtrs bases,
                                                        uint8_t *__restrict__ packed, SumCtx cx)
{
    constexpr uint32_t T = transpose_tile(sizeof(E)), V = 16 / sizeof(E);
    __shared__ __attribute__((aligned(16))) uint8_t lds_raw[T * (T + 1) * sizeof(E)];
    const Tile t = tiles[blockIdx.x];
    uint8_t *user = bases.p[t.tensor] + t.src_off;
    uint8_t *pk = packed + t.packed_off;
    const uint32_t ni = t.n0, nj = t.n1;
    uint64_t acc = 0;
    const uint32_t es = t.estep;                       // tensor side: bytes from element i to element i + 1 (sizeof(E) or more)
    const bool vec_ok = es == sizeof(E) && ((ni | nj) % V) == 0 && ((reinterpret_cast<uintptr_t>(pk) | t.a | t.b) % 16) == 0;
    if (vec_ok) {
        // storage: nj rows (pitch a) of ni contiguous elements; packed: ni rows (pitch b) of nj elements.  Every
        // storage row of the tile is off a 16-byte boundary by the same amount (the pitch is a multiple of 16).
        auto run = [&]<int UA, bool FULL = false>() {
            const PitchRows rows{pk, t.b};
            if constexpr (!UNPACK) return transpose_vec<E, false, CSUM, NTP, UA, FULL>(user, t.a, nj, ni, rows, lds_raw);
            else return transpose_vec<E, true, CSUM, NTP, UA, FULL>(user, t.a, ni, nj, rows, lds_raw);
        };
        const uint32_t mis = uint32_t(reinterpret_cast<uintptr_t>(user)) & 15u;
        if (mis == 0 && ni == T && nj == T) acc = run.template operator()<16, true>();      // the common case
        else if (mis == 0) acc = run.template operator()<16>();
        else if ((mis & 3u) == 0) acc = run.template operator()<4>();
        else if ((mis & 1u) == 0) acc = run.template operator()<2>();
        else acc = run.template operator()<1>();
    } else {
        // Element by element (extents or pitches that are not multiples of 16 bytes, or a tensor side whose
        // fast direction has a stride of a few elements instead of one).  Eight global loads
        // per thread are issued before the first of them is needed (the row number is clamped into the
        // tile, so the loads need no guard of their own).
        E(*lds)[T + 1] = reinterpret_cast<E(*)[T + 1]>(lds_raw);
        const uint32_t tx = threadIdx.x & (T - 1), ty = threadIdx.x / T;
        constexpr uint32_t TY = kThreads / T, U = 8;
        if constexpr (!UNPACK) {
            if (tx < ni)
                for (uint32_t j0 = ty; j0 < nj; j0 += TY * U) {
                    E v[U];
#pragma unroll
                    for (uint32_t u = 0; u < U; ++u)
                        v[u] = __builtin_nontemporal_load(reinterpret_cast<const E *>(user + uint64_t(min(j0 + u * TY, nj - 1)) * t.a + tx * es));
#pragma unroll
                    for (uint32_t u = 0; u < U; ++u)
                        if (j0 + u * TY < nj) lds[j0 + u * TY][tx] = v[u];
                }
            __syncthreads();
            if (tx < nj)
                for (uint32_t i = ty; i < ni; i += TY) {
                    const E v = lds[tx][i];
                    const uint64_t pos = i * t.b + tx * sizeof(E);
                    store_elem<NTP>(reinterpret_cast<E *>(pk + pos), v);
                    if constexpr (CSUM) acc += elem_weighted(v, t.packed_off + pos);
                }
        } else {
            if (tx < nj)
                for (uint32_t i0 = ty; i0 < ni; i0 += TY * U) {
                    E v[U];
#pragma unroll
                    for (uint32_t u = 0; u < U; ++u)
                        v[u] = load_elem<NTP>(reinterpret_cast<const E *>(pk + uint64_t(min(i0 + u * TY, ni - 1)) * t.b + tx * sizeof(E)));
#pragma unroll
                    for (uint32_t u = 0; u < U; ++u) {
                        const uint32_t i = i0 + u * TY;
                        if (i < ni) {
                            lds[tx][i] = v[u];
                            if constexpr (CSUM) acc += elem_weighted(v[u], t.packed_off + i * t.b + tx * sizeof(E));
                        }
                    }
                }
            __syncthreads();
            if (tx < ni)
                for (uint32_t j = ty; j < nj; j += TY)
                    __builtin_nontemporal_store(lds[j][tx], reinterpret_cast<E *>(user + j * t.a + tx * es));
        }
    }
    if constexpr (CSUM) chunk_commit(acc, t.chunk, t.ordinal, chunk_tiles[t.chunk], cx);
}

// ---- transpose whose tiles span chunks -------------------------------------------
// For matrices whose packed rows are long against the chunk: a tile is a full block of the logical matrix
// (so that every memory burst of the tensor side is used whole) and row i of it starts at stream byte
// s0 + i * b, wherever that falls; a tile row is shorter than a chunk, so it meets at most one chunk
// border.  Thread i first places row i (its chunk, the packed address of its first byte, how many of its
// columns lie before the border and where the rest go) and leaves that in LDS, so that the copy loop only
// reads it back.  Checksums are taken on the tensor side, where a thread holds elements of one row only, and
// added to the tile's per-chunk partial sums in LDS; at the end one thread per chunk touched makes that
// chunk's arrival (inc holds the tile's chunks, ascending, and the ordinal of each arrival).
template <typename E, bool UNPACK, bool CSUM, bool NTP>
__global__ __launch_bounds__(kThreads) void k_transpose_span(const Tile *__restrict__ tiles,
                                                             const uint32_t *__restrict__ chunk_tiles,
                                                             const uint32_t *__restrict__ inc, ChunkGeom g,
                                                             BasePtrs bases, uint8_t *__restrict__ packed, SumCtx cx)
{
    constexpr uint32_t T = transpose_tile(sizeof(E));
    constexpr uint32_t TY = kThreads / T, MAXC = 2 * T + 2;
    static_assert(T <= kThreads, "one thread places one row");
    __shared__ __attribute__((aligned(16))) uint8_t lds_raw[T * (T + 1) * sizeof(E)];
    __shared__ unsigned long long part[MAXC];          // partial sum per chunk touched
    __shared__ uint32_t touched[MAXC];                 // those chunks
    // per row: packed offset of column j is row_p0 + j * sizeof(E) for j < row_first, row_p1 + j * sizeof(E) from there on
    __shared__ uint64_t row_p0[T], row_p1[T];
    __shared__ uint32_t row_first[T], row_at[T], row_low[T];   // row_at: entry of the row's first chunk; row_low: low bits of
                                                               // its first byte's position (for the weights of the sum)
    const Tile t = tiles[blockIdx.x];
    uint8_t *user = bases.p[t.tensor] + t.src_off;
    const uint32_t ni = t.n0, nj = t.n1, es = t.estep, n_inc = t.ordinal;
    const uint32_t *my = inc + 2 * size_t(t.chunk);
    E(*lds)[T + 1] = reinterpret_cast<E(*)[T + 1]>(lds_raw);
    const uint32_t tx = threadIdx.x & (T - 1);
    const uint32_t ty = threadIdx.x / T;
    for (uint32_t i = threadIdx.x; i < n_inc; i += kThreads) {
        touched[i] = my[2 * i];
        part[i] = 0;
    }
    __syncthreads();
    if (threadIdx.x < ni) {                             // place row threadIdx.x
        const uint64_t B = g.B, s = t.packed_off + uint64_t(threadIdx.x) * t.b;
        const uint64_t c = s / B, rem = s - c * B;
        uint32_t lo = 0, hi = n_inc - 1;                // the entry that names chunk c (it is there)
        while (lo < hi) {
            const uint32_t mid = (lo + hi) / 2;
            if (touched[mid] < uint32_t(c)) lo = mid + 1;
            else hi = mid;
        }
        auto chunk_base = [&](uint64_t ch) {
            const uint32_t slot = fast_div(uint32_t(ch), g.div_k), lane = uint32_t(ch) - slot * g.k;
            return (uint64_t(lane) * g.q + (lane < g.r ? lane : g.r) + slot) * B;
        };
        const uint64_t room = B - rem;                  // bytes of chunk c from the row's start on
        const uint32_t first = room >= uint64_t(nj) * sizeof(E) ? nj : uint32_t(room / sizeof(E));
        row_at[threadIdx.x] = lo;
        row_first[threadIdx.x] = first;
        row_low[threadIdx.x] = uint32_t(rem) & 3u;
        row_p0[threadIdx.x] = chunk_base(c) + rem;
        row_p1[threadIdx.x] = first < nj ? chunk_base(c + 1) + rem - B : 0;     // (+ j * sizeof(E) >= B - rem for those columns)
    }
    __syncthreads();
    // The tensor side of the tile: thread (tx, ty) moves columns ty, ty + TY, ... of row tx between the tensor and
    // LDS, and while it holds them adds them to the row's sums (the part before the chunk border and the part
    // after it), which go to the tile's per-chunk partial sums: no reduction across lanes.
    constexpr uint32_t U = 8;
    auto tensor_side = [&]() {
        if (tx >= ni) return;
        const uint32_t first = row_first[tx], low = row_low[tx];
        unsigned long long a0 = 0, a1 = 0;
        auto count = [&](E v, uint32_t j) {
            const unsigned long long w = elem_weighted(v, uint64_t(low) + uint64_t(j) * sizeof(E));
            if (j < first) a0 += w;
            else a1 += w;
        };
        if constexpr (!UNPACK) {
            for (uint32_t j0 = ty; j0 < nj; j0 += TY * U) {
                E v[U];
#pragma unroll
                for (uint32_t u = 0; u < U; ++u)
                    v[u] = __builtin_nontemporal_load(reinterpret_cast<const E *>(user + uint64_t(min(j0 + u * TY, nj - 1)) * t.a + tx * es));
#pragma unroll
                for (uint32_t u = 0; u < U; ++u)
                    if (j0 + u * TY < nj) {
                        lds[j0 + u * TY][tx] = v[u];
                        if constexpr (CSUM) count(v[u], j0 + u * TY);
                    }
            }
        } else {
            for (uint32_t j = ty; j < nj; j += TY) {
                const E v = lds[j][tx];
                __builtin_nontemporal_store(v, reinterpret_cast<E *>(user + j * t.a + tx * es));
                if constexpr (CSUM) count(v, j);
            }
        }
        if constexpr (CSUM) {
            const uint32_t at = row_at[tx];
            if (a0) __hip_atomic_fetch_add(&part[at], a0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            if (a1) __hip_atomic_fetch_add(&part[at + 1], a1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
    };
    // The packed side, rows ty, ty + TY, ...: pack stores what is in LDS, unpack fills it.  The loads of an unpack
    // need no guard (a row beyond the tile repeats the last one, lanes beyond its width shadow its last column),
    // so all U of a round are in flight before the first is used.
    auto packed_side = [&]() {
        const uint32_t txc = min(tx, nj - 1);
        for (uint32_t i0 = ty; i0 < ni; i0 += TY * U) {
            E *p[U];
            E v[U];
#pragma unroll
            for (uint32_t u = 0; u < U; ++u) {
                const uint32_t i = min(i0 + u * TY, ni - 1);
                const uint64_t off = (txc < row_first[i] ? row_p0[i] : row_p1[i]) + uint64_t(txc) * sizeof(E);
                p[u] = reinterpret_cast<E *>(packed + off);
                if constexpr (UNPACK) v[u] = load_elem<NTP>(p[u]);
            }
#pragma unroll
            for (uint32_t u = 0; u < U; ++u) {
                const uint32_t i = i0 + u * TY;
                if (i < ni && tx < nj) {
                    if constexpr (UNPACK) lds[tx][i] = v[u];
                    else store_elem<NTP>(p[u], lds[tx][i]);
                }
            }
        }
    };
    // 16-byte vectors on both sides when every extent, pitch and row start allows it (then a row's chunk border
    // falls between two vectors too); the tensor side may be less than 16-byte aligned as a whole.
    constexpr uint32_t V = 16 / sizeof(E);
    const bool vec_ok = es == sizeof(E) && ((ni | nj) % V) == 0 && ((t.packed_off | t.a | t.b) % 16) == 0;
    if (vec_ok) {
        const SpanRows rows{packed, row_p0, row_p1, row_first, row_at, part};    // row_first in bytes: see below
        if (threadIdx.x < ni) row_first[threadIdx.x] *= uint32_t(sizeof(E));     // (its own entry: no other thread reads it yet)
        __syncthreads();
        auto run = [&]<int UA, bool FULL = false>() {
            if constexpr (!UNPACK) transpose_vec<E, false, CSUM, NTP, UA, FULL>(user, t.a, nj, ni, rows, lds_raw);
            else transpose_vec<E, true, CSUM, NTP, UA, FULL>(user, t.a, ni, nj, rows, lds_raw);
        };
        const uint32_t mis = uint32_t(reinterpret_cast<uintptr_t>(user)) & 15u;
        if (mis == 0 && ni == T && nj == T) run.template operator()<16, true>();
        else if (mis == 0) run.template operator()<16>();
        else if ((mis & 3u) == 0) run.template operator()<4>();
        else if ((mis & 1u) == 0) run.template operator()<2>();
        else run.template operator()<1>();
    } else if constexpr (!UNPACK) {
        tensor_side();
        __syncthreads();
        packed_side();
    } else {
        packed_side();
        __syncthreads();
        tensor_side();
    }
    if constexpr (CSUM) {
        __syncthreads();
        for (uint32_t i = threadIdx.x; i < n_inc; i += kThreads)
            commit_total(part[i], touched[i], my[2 * i + 1], chunk_tiles[touched[i]], cx);
    }
}

// ---- generic: any strides, one element at a time -------------------------------
// Every element's address is recomputed from its logical index.  Only used for views the
// other kernels do not take (no dimension with stride one, or runs shorter than 16 bytes).
// The elements [e0, e0 + nel) of one tensor, every dim within reach of the multiply-shift division.
// ND > 0: the tensor has exactly ND merged dims; ND == 0: any number, read from the descriptor.
// The dims are copied into registers first: the loop below stores through byte pointers, which
// may alias anything, so values read through the descriptor inside it would be read again for
// every element.  Consecutive lanes take consecutive elements, U of them in flight per thread:
// a wave's access is contiguous on the packed side and as dense on the tensor side as the view
// allows.  The loads of a round are unconditional (the index is clamped into the tile), so that
// all of them are issued before the first is waited for; only the stores are guarded.
template <typename E, bool UNPACK, bool CSUM, bool NTP, int ND>
__device__ __forceinline__ uint64_t generic_span(const TensorDev &td, uint64_t e0, uint32_t nel, uint8_t *user, E *p)
{
    constexpr int D = ND ? ND : HXT_MAX_DIMS;
    const int nd = ND ? ND : td.ndim;
    uint32_t shape[D], mul[D], shift[D], first[D];
    uint64_t stride[D];
    {
        uint64_t idx = e0;                                  // coordinates of the span's first element
#pragma unroll
        for (int d = D - 1; d >= 0; --d) {
            shape[d] = 1, mul[d] = 0, shift[d] = 0, first[d] = 0, stride[d] = 0;
            if (d < nd) {
                shape[d] = uint32_t(td.shape[d]);
                mul[d] = td.dim_div[d].mul;
                shift[d] = td.dim_div[d].shift;
                stride[d] = uint64_t(td.stride_b[d]);
                const uint64_t q = idx / uint64_t(td.shape[d]);
                first[d] = uint32_t(idx - q * uint64_t(td.shape[d]));
                idx = q;
            }
        }
    }
    // An element's coordinates are the first element's plus its number within the span, carried from
    // the last dim upwards in 32 bits (a span has fewer than 2^30 elements and so has every dim).
    auto locate = [&](uint32_t el) -> E * {
        uint64_t off = 0;
        uint32_t x = el;
#pragma unroll
        for (int d = D - 1; d > 0; --d) {
            if (d < nd) {
                x += first[d];
                const uint32_t q = fast_div(x, FastDiv{mul[d], shift[d]});
                off += uint64_t(x - q * shape[d]) * stride[d];
                x = q;
            }
        }
        off += uint64_t(x + first[0]) * stride[0];
        return reinterpret_cast<E *>(user + off);
    };
    constexpr int U = 8;
    uint64_t acc = 0;
    const uint32_t last = nel - 1;
    for (uint32_t e1 = threadIdx.x; e1 < nel; e1 += kThreads * U) {
        E val[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t el = min(e1 + u * kThreads, last);
            if constexpr (UNPACK) val[u] = load_elem<NTP>(p + el);
            else val[u] = load_elem<true>(locate(el));
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t el = e1 + u * kThreads;
            if (el < nel) {
                if constexpr (UNPACK) store_elem<true>(locate(el), val[u]);
                else store_elem<NTP>(p + el, val[u]);
                if constexpr (CSUM) acc += elem_weighted(val[u], uint64_t(el) * sizeof(E));
            }
        }
    }
    return acc;
}

// The same for tensors with a dim beyond the reach of the multiply-shift division: every element's
// index is divided out in 64 bits.
template <typename E, bool UNPACK, bool CSUM, bool NTP>
__device__ __noinline__ uint64_t generic_span_wide(const TensorDev &td, uint64_t e0, uint32_t nel, uint8_t *user, E *p)
{
    const int nd = td.ndim;
    uint64_t acc = 0;
    for (uint32_t el = threadIdx.x; el < nel; el += kThreads) {
        uint64_t idx = e0 + el, off = 0;
        for (int d = nd - 1; d >= 0; --d) {
            const uint64_t q = idx / uint64_t(td.shape[d]);
            off += (idx - q * uint64_t(td.shape[d])) * uint64_t(td.stride_b[d]);
            idx = q;
        }
        E *at = reinterpret_cast<E *>(user + off);
        E v;
        if constexpr (UNPACK) {
            v = load_elem<NTP>(p + el);
            store_elem<true>(at, v);
        } else {
            v = load_elem<true>(at);
            store_elem<NTP>(p + el, v);
        }
        if constexpr (CSUM) acc += elem_weighted(v, uint64_t(el) * sizeof(E));
    }
    return acc;
}

template <typename E, bool UNPACK, bool CSUM, bool NTP>
__global__ __launch_bounds__(kThreads) void k_generic(const Tile *__restrict__ tiles,
                                                      const uint32_t *__restrict__ chunk_tiles,
                                                      const TensorDev *__restrict__ tensors, uint32_t tensor_base,
                                                      BasePtrs bases, uint8_t *__restrict__ packed, SumCtx cx)
{
    const Tile t = tiles[blockIdx.x];
    uint64_t acc = 0;
    if (t.kind == K_ZERO) {
        acc = pad_span<UNPACK, CSUM>(packed + t.packed_off, t.n0, uint32_t(t.packed_off));
    } else {
        const TensorDev &td = tensors[tensor_base + t.tensor];
        uint8_t *user = bases.p[t.tensor];
        E *p = reinterpret_cast<E *>(packed + t.packed_off);
        const uint32_t nel = t.n0 / sizeof(E);
        const uint64_t e0 = t.src_off / sizeof(E);
        if (nel == 0) {
        } else if (!td.all_div) {
            acc = generic_span_wide<E, UNPACK, CSUM, NTP>(td, e0, nel, user, p);
        } else {
            switch (td.ndim) {
            case 1: acc = generic_span<E, UNPACK, CSUM, NTP, 1>(td, e0, nel, user, p); break;
            case 2: acc = generic_span<E, UNPACK, CSUM, NTP, 2>(td, e0, nel, user, p); break;
            case 3: acc = generic_span<E, UNPACK, CSUM, NTP, 3>(td, e0, nel, user, p); break;
            case 4: acc = generic_span<E, UNPACK, CSUM, NTP, 4>(td, e0, nel, user, p); break;
            default: acc = generic_span<E, UNPACK, CSUM, NTP, 0>(td, e0, nel, user, p); break;
            }
        }
    }
    if constexpr (CSUM) chunk_commit(acc, t.chunk, t.ordinal, chunk_tiles[t.chunk], cx);
}

// ---- stand-alone checksum of packed chunks (closed-form geometry, no table) ----------
template <bool NTP>
__global__ __launch_bounds__(kThreads) void k_checksum(ChunkGeom g, const uint8_t *__restrict__ packed, SumCtx cx)
{
    const TileSpan t = locate_tile(g, blockIdx.x);
    const u32x4 *s = reinterpret_cast<const u32x4 *>(packed + t.packed_off);
    const uint32_t nvec = t.len >> 4;
    uint64_t acc = 0;
    for (uint32_t v = threadIdx.x; v < nvec; v += kThreads * kUnroll) {
        u32x4 r[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
            r[u] = load16_or_zero<NTP>(s, v + u * kThreads, nvec);
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) acc += words_sum(r[u]);
    }
    chunk_commit(acc, t.chunk, t.ordinal, t.expected, cx);
}

// ---- stand-alone strong check: plain sum and position-weighted sum of every chunk -------
// out[2c] = sum of the chunk's words, out[2c+1] = sum of (j+1) * word j, both mod 2^64.
// A logical accumulator is a pair of slots (2s: plain sum and arrival count, 2s+1: weighted
// sum); the ticket is taken after both additions have returned.  Same two-level fan-out as
// chunk_commit: first-level pairs C*fan, then one second-level pair per chunk.
// sum_bits > 0 (see slot_arrive): the plain sum and the arrival count share one word, so the arrival is
// the weighted sum's addition, then one addition that also takes the ticket; sum_bits == 0: three steps.
__device__ __forceinline__ bool pair_arrive(uint8_t *acc, uint32_t stride, size_t s, unsigned long long &a,
                                            unsigned long long &b, uint32_t expected, uint32_t sum_bits)
{
    if (expected == 1) return true;
    Acc *sa = reinterpret_cast<Acc *>(acc + (2 * s) * stride);
    Acc *sb = reinterpret_cast<Acc *>(acc + (2 * s + 1) * stride);
    const unsigned long long rb = __hip_atomic_fetch_add(&sb->sum, b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (sum_bits) {
        asm volatile("s_waitcnt vmcnt(0)" ::"v"(uint32_t(rb)) : "memory");
        const unsigned long long one = 1ull << sum_bits;
        const unsigned long long before = __hip_atomic_fetch_add(&sa->sum, one + a, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((before >> sum_bits) != expected - 1) return false;
        __hip_atomic_store(&sa->sum, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        a = (before + a) & (one - 1);
        b = __hip_atomic_exchange(&sb->sum, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return true;
    }
    const unsigned long long ra = __hip_atomic_fetch_add(&sa->sum, a, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("s_waitcnt vmcnt(0)" ::"v"(uint32_t(ra)), "v"(uint32_t(rb)) : "memory");
    const uint32_t ticket = __hip_atomic_fetch_add(&sa->cnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (ticket != expected - 1) return false;
    a = __hip_atomic_exchange(&sa->sum, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    b = __hip_atomic_exchange(&sb->sum, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(&sa->cnt, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return true;
}

// Word j of the chunk sits at tile word i = j - j0.  A thread's vectors start at tile words
// 4 * (tid + 256 * n), n = 0, 1, ...; with S_n the sum of vector n's words and I_n = y + 2z + 3w,
//   sum (j+1) w_j = (j0 + 4 tid + 1) * sum_n S_n + 1024 * sum_n n S_n + sum_n I_n,
// so the loop needs additions only (sum_n n S_n is kept as a running suffix sum) and each
// thread multiplies once.
//
// MODE says what the workgroup that completes a chunk does with the two sums:
//   SUMS   out = uint64[2C]: writes the pair.
//   SEAL   out = C tags: writes the chunk's 64-byte tag (hxt_chunk_tag_t) at its packed-slot index.
//   VERIFY out = uint32[C + 1], tags = C tags: compares the tag found at the chunk's slot with the
//          receiver's own layout, the expected message identity and the recomputed sums, and
//          writes the bit mask to out[chunk].
enum Sum2Mode { SUM2_SUMS = 0, SUM2_SEAL = 1, SUM2_VERIFY = 2 };

struct TagWork {
    const uint8_t *tags;     // VERIFY: the received tags
    uint64_t seq;            // SEAL: value to write; VERIFY: value expected
    uint32_t micro_batch;
    uint32_t sum_bits;       // see pair_arrive; set by the launch code
};

// The received tag of a workgroup's chunk, loaded by thread 0 when the workgroup starts so that the load's
// latency is long past when (and if) this workgroup turns out to complete the chunk.
struct TagRegs {
    u32x4 r[4];
};

__device__ __forceinline__ uint64_t tag_place(const ChunkGeom &g, uint32_t c)     // packed offset of chunk c / B
{
    const uint32_t slot = fast_div(c, g.div_k), lane = c - slot * g.k;
    return uint64_t(lane) * g.q + (lane < g.r ? lane : g.r) + slot;
}

__device__ __forceinline__ TagRegs prefetch_tag(int mode, const ChunkGeom &g, uint32_t chunk, const TagWork &w)
{
    TagRegs t{};
    if (mode == SUM2_VERIFY && threadIdx.x == 0) {
        const u32x4 *tag = reinterpret_cast<const u32x4 *>(w.tags + tag_place(g, chunk) * 64);
#pragma unroll
        for (int i = 0; i < 4; ++i) t.r[i] = tag[i];
    }
    return t;
}

__device__ __forceinline__ void finish_chunk(int mode, const ChunkGeom &g, const TileSpan &t, uint64_t sum,
                                             uint64_t wsum, void *out, const TagWork &w, const TagRegs &got,
                                             uint8_t *acc, uint32_t stride, uint32_t fan)
{
    const uint32_t c = t.chunk;
    if (mode == SUM2_SUMS) {
        uint64_t *o = static_cast<uint64_t *>(out);
        o[2 * size_t(c)] = sum;
        o[2 * size_t(c) + 1] = wsum;
        return;
    }
    const uint32_t slot = fast_div(c, g.div_k), lane = c - slot * g.k;
    const uint64_t place = tag_place(g, c);
    const uint64_t padded = (c + 1 == g.C) ? g.L - uint64_t(c) * g.B : g.B;
    const u32x4 q0{kTagMagic, c, lane, slot};
    const u32x4 q1{uint32_t(w.seq), uint32_t(w.seq >> 32), w.micro_batch, g.C};
    const u32x4 q2{uint32_t(padded), uint32_t(padded >> 32), uint32_t(sum), uint32_t(sum >> 32)};
    const u32x4 q3{uint32_t(wsum), uint32_t(wsum >> 32), 0u, 0u};
    if (mode == SUM2_SEAL) {
        u32x4 *tag = reinterpret_cast<u32x4 *>(static_cast<uint8_t *>(out) + place * 64);
        tag[0] = q0;
        tag[1] = q1;
        tag[2] = q2;
        tag[3] = q3;
        return;
    }
    const u32x4 r0 = got.r[0], r1 = got.r[1], r2 = got.r[2], r3 = got.r[3];
    uint32_t m = 0;
    if (r0.x != q0.x) m |= HXT_TAG_BAD_MAGIC;
    if (r0.y != q0.y || r0.z != q0.z || r0.w != q0.w || r1.w != q1.w || r2.x != q2.x || r2.y != q2.y) m |= HXT_TAG_BAD_PLACE;
    if (r1.x != q1.x || r1.y != q1.y) m |= HXT_TAG_BAD_SEQ;
    if (r1.z != q1.z) m |= HXT_TAG_BAD_MICRO_BATCH;
    if (r2.z != q2.z || r2.w != q2.w) m |= HXT_TAG_BAD_SUM;
    if (r3.x != q3.x || r3.y != q3.y) m |= HXT_TAG_BAD_WSUM;
    if (r3.z != 0 || r3.w != 0) m |= HXT_TAG_BAD_RESERVED;
    static_cast<uint32_t *>(out)[c] = m;
    // One more slot, after the chunks' own pairs, counts the chunks that are done (upper half of the word)
    // and the rejected ones among them (lower half) with one addition; the chunk that completes the
    // message writes the total to out[C] and clears the slot.
    const unsigned long long mine = (1ull << 32) | (m != 0 ? 1u : 0u);
    unsigned long long total = mine;
    if (g.C > 1) {
        Acc *done = reinterpret_cast<Acc *>(acc + 2 * (size_t(g.C) * (fan + 1)) * stride);
        const unsigned long long before = __hip_atomic_fetch_add(&done->sum, mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (uint32_t(before >> 32) != g.C - 1) return;
        __hip_atomic_store(&done->sum, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        total = before + mine;
    }
    static_cast<uint32_t *>(out)[g.C] = uint32_t(total);
}

// Workgroup-wide: reduces every thread's (a, b), adds the pair to the chunk's accumulators (two-level
// fan-out as in chunk_commit); the workgroup that completes the chunk finishes it.
__device__ __forceinline__ void pair_commit(int mode, const ChunkGeom &g, const TileSpan &t, unsigned long long a,
                                            unsigned long long b, void *out, uint8_t *acc, uint32_t stride,
                                            uint32_t fan, const TagWork &work, const TagRegs &got)
{
    __shared__ uint64_t part[2][kThreads / 64];
    for (int o = 32; o > 0; o >>= 1) {
        a += __shfl_down(a, o, 64);
        b += __shfl_down(b, o, 64);
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) {
        part[0][wave] = a;
        part[1][wave] = b;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        a = b = 0;
#pragma unroll
        for (int w = 0; w < kThreads / 64; ++w) {
            a += part[0][w];
            b += part[1][w];
        }
        const size_t top = size_t(g.C) * fan + t.chunk;
        bool last;
        if (fan == 1 || t.expected < 2 * fan) {
            last = pair_arrive(acc, stride, top, a, b, t.expected, work.sum_bits);
        } else {
            const uint32_t sub = t.ordinal & (fan - 1);
            const uint32_t share = t.expected / fan + (sub < (t.expected & (fan - 1)) ? 1u : 0u);
            last = pair_arrive(acc, stride, size_t(t.chunk) * fan + sub, a, b, share, work.sum_bits) &&
                   pair_arrive(acc, stride, top, a, b, fan, work.sum_bits);
        }
        if (last) finish_chunk(mode, g, t, a, b, out, work, got, acc, stride, fan);
    }
}

template <int MODE, bool NTP>
__global__ __launch_bounds__(kThreads) void k_checksum2(ChunkGeom g, const uint8_t *__restrict__ packed,
                                                        void *__restrict__ out, uint8_t *acc, uint32_t stride,
                                                        uint32_t fan, TagWork work)
{
    const TileSpan t = locate_tile(g, blockIdx.x);
    const TagRegs got = prefetch_tag(MODE, g, t.chunk, work);
    const u32x4 *s = reinterpret_cast<const u32x4 *>(packed + t.packed_off);
    const uint64_t j0 = (t.stream_off - uint64_t(t.chunk) * g.B) >> 2;
    const uint32_t nvec = t.len >> 4;
    uint64_t S = 0, nS = 0, I = 0;          // sum_n S_n, sum_n n*S_n, sum_n I_n
    uint64_t n0 = 0;                         // n of the current block of vectors
    for (uint32_t v = threadIdx.x; v < nvec; v += kThreads * kUnroll, n0 += kUnroll) {
        u32x4 r[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
            r[u] = load16_or_zero<NTP>(s, v + u * kThreads, nvec);
        uint64_t blockS = 0, blockN = 0;     // this block's sum_u S_u and sum_u u*S_u
#pragma unroll
        for (int u = kUnroll - 1; u >= 0; --u) {
            const uint64_t zw = uint64_t(r[u].z) + r[u].w;
            const uint64_t yzw = zw + r[u].y;
            blockN += blockS;                // after the loop: sum_u u * S_u
            blockS += yzw + r[u].x;
            I += yzw + zw + r[u].w;
        }
        S += blockS;
        nS += blockN + n0 * blockS;
    }
    pair_commit(MODE, g, t, S, (j0 + 4ull * threadIdx.x + 1) * S + 4ull * kThreads * nS + I, out, acc, stride, fan, work, got);
}

// ---- pack + seal and unpack + verify in one pass (messages that are one contiguous tensor) ----
// The copy of k_uniform with both sums of the packed words taken on the way, so that tags cost no
// extra pass over the message.  Weights are tile-local here (word i of the tile weighs i + 1);
// the tile's position in its chunk is applied once per workgroup.
struct Sums2 {
    uint64_t s, w;
};

// A thread's vectors are numbers tid + 256 n (n = 0, 1, ...) of the tile; with S_n the sum of vector n's words and
// I_n = y + 2z + 3w, the tile-local weighted sum is
//   sum (i + 1) w_i = (4 tid + 1) * sum_n S_n + 1024 * sum_n n S_n + sum_n I_n,
// so the loop only adds (as in k_checksum2) and each thread multiplies once at the end.
struct Partial2 {
    uint64_t S, nS, I;
    __device__ __forceinline__ void add(u32x4 r, uint64_t n)
    {
        const uint64_t zw = uint64_t(r.z) + r.w, yzw = zw + r.y, sv = yzw + r.x;
        S += sv;
        nS += n * sv;
        I += yzw + zw + r.w;
    }
};

template <bool UNPACK, bool NTU, bool NTP>
__device__ __forceinline__ Sums2 copy_span2(uint8_t *user, uint8_t *pk, uint32_t bytes)
{
    constexpr bool NTL = UNPACK ? NTP : NTU, NTS = UNPACK ? NTU : NTP;
    const u32x4 *s = reinterpret_cast<const u32x4 *>(UNPACK ? pk : user);
    u32x4 *d = reinterpret_cast<u32x4 *>(UNPACK ? user : pk);
    const uint32_t nvec = bytes >> 4;
    constexpr uint32_t STEP = kThreads * kUnroll;
    const uint32_t full = nvec / STEP * STEP;
    Partial2 p{0, 0, 0};
    uint64_t n0 = 0;                                     // n of the current block's first vector
    uint32_t v = threadIdx.x;
    for (; v < full; v += STEP, n0 += kUnroll) {
        u32x4 r[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) r[u] = load16<NTL>(s + v + u * kThreads);
        uint64_t blockS = 0, blockN = 0, blockI = 0;     // this block's sum_u S_u, sum_u u * S_u, sum_u I_u
#pragma unroll
        for (int u = kUnroll - 1; u >= 0; --u) {
            store16<NTS>(d + v + u * kThreads, r[u]);
            const uint64_t zw = uint64_t(r[u].z) + r[u].w, yzw = zw + r[u].y;
            blockN += blockS;                            // after the loop: sum_u u * S_u
            blockS += yzw + r[u].x;
            blockI += yzw + zw + r[u].w;
        }
        p.S += blockS;
        p.nS += blockN + n0 * blockS;
        p.I += blockI;
    }
    for (; v < nvec; v += kThreads, ++n0) {
        const u32x4 r = load16<NTL>(s + v);
        store16<NTS>(d + v, r);
        p.add(r, n0);
    }
    Sums2 acc{p.S, uint64_t(4 * threadIdx.x + 1) * p.S + 4ull * kThreads * p.nS + p.I};
    const uint32_t tail = bytes & 15;                    // only at the very end of the tensor
    if (threadIdx.x < tail) {
        const uint32_t i = (nvec << 4) + threadIdx.x;
        const uint8_t b = (UNPACK ? pk : user)[i];
        (UNPACK ? user : pk)[i] = b;
        const uint64_t val = uint64_t(b) << (8 * (i & 3));
        acc.s += val;
        acc.w += uint64_t((i >> 2) + 1) * val;
    }
    return acc;
}

// Pad bytes after the tensor's last byte, `first` = their byte position in the tile: pack writes zeros
// (which add nothing to either sum), unpack adds what it finds there.
template <bool UNPACK>
__device__ __forceinline__ Sums2 pad_span2(uint8_t *pk, uint32_t bytes, uint64_t first)
{
    Sums2 acc{0, 0};
    for (uint32_t i = threadIdx.x; i < bytes; i += kThreads) {
        if constexpr (!UNPACK) {
            pk[i] = 0;
        } else {
            const uint64_t pos = first + i;
            const uint64_t val = uint64_t(pk[i]) << (8 * (pos & 3));
            acc.s += val;
            acc.w += uint64_t((pos >> 2) + 1) * val;
        }
    }
    return acc;
}

// One launch serves up to kMaxBatch such messages (workgroups [first_tile, first_tile + ntiles) belong to
// message i), as k_uniform does for the plain sums.
struct UniformTagItem {
    ChunkGeom g;
    uint8_t *user;
    uint8_t *packed;
    void *out;             // SEAL: the message's tags; VERIFY: its status words
    uint8_t *acc;          // the plan's pair-of-sums accumulator slots
    uint32_t stride, fan;
    TagWork work;
    uint32_t first_tile;
};

struct UniformTagArgs {
    UniformTagItem it[kMaxBatch];
    uint32_t n;
};

template <bool UNPACK, int MODE, bool NTU, bool NTP>
__global__ __launch_bounds__(kThreads) void k_uniform_tag(UniformTagArgs a)
{
    uint32_t m = 0;
#pragma unroll
    for (uint32_t i = 1; i < kMaxBatch; ++i)
        if (i < a.n && blockIdx.x >= a.it[i].first_tile) m = i;
    const UniformTagItem &it = a.it[m];
    const ChunkGeom &g = it.g;
    const TileSpan t = locate_tile(g, blockIdx.x - it.first_tile);
    const TagRegs got = prefetch_tag(MODE, g, t.chunk, it.work);
    const uint64_t left = g.N > t.stream_off ? g.N - t.stream_off : 0;
    const uint32_t data = left < t.len ? uint32_t(left) : t.len;
    uint8_t *pk = it.packed + t.packed_off;
    Sums2 sums = copy_span2<UNPACK, NTU, NTP>(it.user + t.stream_off, pk, data);
    if (data < t.len) {
        const Sums2 pad = pad_span2<UNPACK>(pk + data, t.len - data, data);
        sums.s += pad.s;
        sums.w += pad.w;
    }
    const uint64_t j0 = (t.stream_off - uint64_t(t.chunk) * g.B) >> 2;       // the tile's first word in its chunk
    pair_commit(MODE, g, t, sums.s, j0 * sums.s + sums.w, it.out, it.acc, it.stride, it.fan, it.work, got);
}

// The same for the contiguous tensors of a multi-tensor message (gradient buckets): the table-driven copy
// of k_contig with both sums taken on the way.  A tile's record says where it starts inside its chunk.
template <bool UNPACK, int MODE, bool NTU, bool NTP>
__global__ __launch_bounds__(kThreads) void k_contig_tag(const Tile *__restrict__ tiles,
                                                         const uint32_t *__restrict__ chunk_tiles, BasePtrs bases,
                                                         uint8_t *__restrict__ packed, ChunkGeom g, void *out,
                                                         uint8_t *acc, uint32_t stride, uint32_t fan, TagWork work)
{
    const Tile t = tiles[blockIdx.x];
    const TagRegs got = prefetch_tag(MODE, g, t.chunk, work);
    TileSpan span{};
    span.chunk = t.chunk;
    span.ordinal = t.ordinal;
    span.expected = chunk_tiles[t.chunk];
    Sums2 sums;
    uint64_t j0 = 0;
    if (t.kind == K_ZERO) {                                  // byte granular: weights taken from the chunk's start
        sums = pad_span2<UNPACK>(packed + t.packed_off, t.n0, t.a);
    } else {
        sums = copy_span2<UNPACK, NTU, NTP>(bases.p[t.tensor] + t.src_off, packed + t.packed_off, t.n0);
        j0 = t.a >> 2;
    }
    pair_commit(MODE, g, span, sums.s, j0 * sums.s + sums.w, out, acc, stride, fan, work, got);
}

// A few KiB of chunk tags between device memory and pinned host memory (either direction; the pinned
// buffer is addressed directly over the host link).  A kernel rather than a DMA copy: a launch costs
// less than the fixed overhead of a copy command, and the DMA queues keep only the large staging copies.
__global__ __launch_bounds__(kThreads) void k_copy_tags(u32x4 *__restrict__ to, const u32x4 *__restrict__ from, uint32_t nvec)
{
    for (uint32_t v = blockIdx.x * kThreads + threadIdx.x; v < nvec; v += gridDim.x * kThreads) to[v] = from[v];
}

// Plain copy of nvec 16-byte vectors by a small grid (grid-stride), for staging between device memory and
// pinned host memory over the host link: a few dozen workgroups keep the link busy and leave the rest of the
// chip to other kernels.  The device side is streamed (non-temporal), four vectors in flight per thread.
__global__ __launch_bounds__(kThreads) void k_stage_copy(u32x4 *__restrict__ to, const u32x4 *__restrict__ from, uint64_t nvec)
{
    const uint64_t step = uint64_t(gridDim.x) * kThreads;
    uint64_t v = uint64_t(blockIdx.x) * kThreads + threadIdx.x;
    for (; v + 3 * step < nvec; v += 4 * step) {
        u32x4 r[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) r[u] = __builtin_nontemporal_load(from + v + u * step);
#pragma unroll
        for (int u = 0; u < 4; ++u) __builtin_nontemporal_store(r[u], to + v + u * step);
    }
    for (; v < nvec; v += step) __builtin_nontemporal_store(__builtin_nontemporal_load(from + v), to + v);
}

// Zero-fill of nvec 16-byte vectors (a kernel, so that it can be recorded where a memset node cannot).
__global__ __launch_bounds__(kThreads) void k_fill_zero(u32x4 *__restrict__ p, uint32_t nvec)
{
    for (uint32_t v = blockIdx.x * kThreads + threadIdx.x; v < nvec; v += gridDim.x * kThreads) p[v] = u32x4{0, 0, 0, 0};
}

// status[C] = number of chunks of status[0 .. C) that were rejected.  One workgroup.
__global__ __launch_bounds__(kThreads) void k_count_rejected(uint32_t *status, uint32_t C)
{
    __shared__ uint32_t part[kThreads / 64];
    uint32_t n = 0;
    for (uint32_t c = threadIdx.x; c < C; c += kThreads) n += status[c] != 0;
    for (int o = 32; o > 0; o >>= 1) n += __shfl_down(n, o, 64);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = n;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t total = 0;
#pragma unroll
        for (int w = 0; w < kThreads / 64; ++w) total += part[w];
        status[C] = total;
    }
}

}  // namespace hxt

#endif
