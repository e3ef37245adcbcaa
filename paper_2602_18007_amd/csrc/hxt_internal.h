// Internal structures shared by the host planner and the HIP kernels of libhxt.
// Not part of the ABI.
#ifndef HXT_INTERNAL_H
#define HXT_INTERNAL_H

#include <cstdint>
#include <vector>

#include "hxt.h"

#if defined(__HIPCC__)
#define HXT_HD __host__ __device__ inline
#else
#define HXT_HD inline
#endif

namespace hxt {

// Which kernel family moves a piece of the stream.
enum Kind : uint16_t {
    K_NONE = 0,
    K_CONTIG = 1,     // tensor bytes are contiguous in memory: straight 128-bit copy
    K_ROWS = 2,       // innermost dimension contiguous, 16-byte friendly rows: gather of runs
    K_TRANSPOSE = 3,  // innermost logical dim strided, second innermost contiguous: LDS tile transpose
    K_GENERIC = 4,    // anything else: one element at a time
    K_ZERO = 5,       // pad bytes between tensors / after the last one (byte granular, < 256 bytes)
    K_ROWS_SPLIT = 6, // innermost dimension contiguous, runs of 16 bytes or more whose length or pitch is not a
                      // multiple of 16: a 16-byte packed vector may end one run and begin the next
    K_TRANSPOSE_SPAN = 7  // the transpose when a chunk holds fewer rows of the packed side than a tile is high: a tile
                          // is a full block of the logical matrix and its rows may lie in different chunks
};

// One unit of work for one workgroup.  64 bytes of 32/64-bit fields, read with scalar loads.
//   linear kinds (CONTIG, ROWS, GENERIC, ZERO):
//     packed_off : first packed byte of the piece (CONTIG/ROWS/GENERIC: multiple of 256)
//     src_off    : logical byte offset inside the tensor (equals the storage offset for CONTIG)
//     n0         : bytes of the piece
//     a          : byte offset of the piece inside its chunk
//   TRANSPOSE (a 2-D block of ni logical rows x nj logical columns inside one chunk):
//     packed_off : packed byte of element (i0, j0);  b = packed row pitch in bytes
//     src_off    : storage byte of element (i0, j0); a = storage pitch between columns in bytes
//     n0 = ni (rows, contiguous in storage), n1 = nj (columns, contiguous in the packed stream)
//   TRANSPOSE_SPAN (the same block, not confined to one chunk): as TRANSPOSE, except
//     packed_off : byte of element (i0, j0) in the logical stream (the kernel finds every row's chunk from it)
//     chunk      : index of the tile's first entry in Plan::inc;  ordinal = number of entries (chunks it touches)
struct Tile {
    uint64_t packed_off;
    uint64_t src_off;
    uint64_t a;
    uint64_t b;
    uint32_t chunk;
    uint32_t tensor;   // index relative to the launch group's first tensor
    uint32_t kind;
    uint32_t n0;
    uint32_t n1;
    uint32_t ordinal;  // position of this tile among the tiles of its chunk (0 .. chunk_tiles[chunk] - 1)
    uint32_t estep;    // TRANSPOSE: bytes between neighbouring elements along the tensor side's fast direction
    uint32_t reserved;
};
static_assert(sizeof(Tile) == 64, "Tile must stay 64 bytes");

// Exact unsigned division of n < 2^31 by a fixed d < 2^31: q = (n * mul) >> (31 + shift).
struct FastDiv {
    uint32_t mul;
    uint32_t shift;
};
FastDiv make_fastdiv(uint32_t d);
HXT_HD uint32_t fast_div(uint32_t n, FastDiv d) { return uint32_t((uint64_t(n) * d.mul) >> (31 + d.shift)); }

// Chunk/lane geometry in closed form, for work that is uniform over the packed stream (a
// message made of one contiguous tensor; the stand-alone checksum of any message).  The
// stream is cut into chunks of B bytes and every chunk into tpc = ceil(B / tile) tiles;
// tile number t belongs to chunk t / tpc.  Lane l holds q + (l < r) chunks, so its region
// starts at (l*q + min(l, r)) * B.
struct ChunkGeom {
    uint64_t N;          // tensor bytes (uniform-copy path only)
    uint64_t L;          // stream bytes (multiple of 256)
    uint64_t B;          // chunk bytes
    uint32_t k, C;       // lanes, chunks
    uint32_t tile;       // bytes per tile (multiple of 256)
    uint32_t tpc;        // tiles per full chunk
    uint32_t q, r;       // C / k, C % k
    uint32_t ntiles;     // (C - 1) * tpc + tiles of the last chunk
    uint32_t last_tiles; // tiles of the last chunk
    FastDiv div_tpc, div_k;
};

struct TileSpan {
    uint32_t chunk;
    uint32_t ordinal;    // position of the tile inside its chunk
    uint32_t expected;   // tiles that make up this chunk
    uint64_t stream_off; // first stream byte of the tile
    uint64_t packed_off; // where it lives in the packed buffer
    uint32_t len;        // stream bytes in the tile (multiple of 256)
};

HXT_HD TileSpan locate_tile(const ChunkGeom &g, uint32_t t)
{
    TileSpan s;
    const uint32_t c = fast_div(t, g.div_tpc), j = t - c * g.tpc;
    const uint32_t slot = fast_div(c, g.div_k), lane = c - slot * g.k;
    const uint64_t in_chunk = uint64_t(j) * g.tile;
    const uint64_t chunk_len = (c + 1 == g.C) ? g.L - uint64_t(c) * g.B : g.B;
    const uint64_t left = chunk_len - in_chunk;
    s.chunk = c;
    s.ordinal = j;
    s.expected = (c + 1 == g.C) ? g.last_tiles : g.tpc;
    s.stream_off = uint64_t(c) * g.B + in_chunk;
    s.packed_off = (uint64_t(lane) * g.q + (lane < g.r ? lane : g.r) + slot) * g.B + in_chunk;
    s.len = left < g.tile ? uint32_t(left) : g.tile;
    return s;
}

// Per-tensor view description for the ROWS and GENERIC kernels (merged dims, logical order).
struct TensorDev {
    int32_t ndim;                      // merged dims; for ROWS the last one is the contiguous run
    int32_t esize;
    uint32_t row_bytes;                // ROWS: bytes of one contiguous run
    uint32_t all_div;                  // 1: dim_div is valid for every dim and every shape[d] <= 2^30
    uint32_t low_or;                   // ROWS_SPLIT: OR of the run length and the outer strides in bytes (their low bits
                                       // give the widest naturally aligned piece the tensor side can be accessed in)
    uint32_t reserved;
    FastDiv row_div;                   // ROWS: division by row_bytes
    FastDiv dim_div[HXT_MAX_DIMS];     // division by shape[d]: for the outer dims of a ROWS tensor, for all dims if all_div
    int64_t shape[HXT_MAX_DIMS];
    int64_t stride_b[HXT_MAX_DIMS];    // bytes
};

constexpr int kMaxGroupTensors = 64;   // base pointers passed by value per launch

struct TensorPlan {
    int ndim = 0;                      // merged
    int64_t shape[HXT_MAX_DIMS] = {0};
    int64_t stride[HXT_MAX_DIMS] = {0};  // elements
    int esize = 1;
    hxt_dtype_t dtype = HXT_U8;
    uint64_t elems = 0, bytes = 0, stream_off = 0;
    Kind kind = K_NONE;
    bool unpack_safe = true;
};

struct Group {          // one kernel launch
    Kind kernel;        // K_CONTIG (serves ZERO tiles too), K_ROWS, K_ROWS_SPLIT, K_TRANSPOSE, K_GENERIC
    uint32_t first;     // first tile
    uint32_t count;
    uint32_t tensor_base;
    uint32_t n_tensors; // tensors addressed: [tensor_base, tensor_base + n_tensors)
};

struct Plan {
    std::vector<TensorPlan> tensors;
    uint64_t N = 0, L = 0, B = 0, C = 0;
    int k = 1;
    std::vector<uint64_t> lane_off;      // k + 1 entries
    std::vector<uint64_t> lane_chunks;   // k
    uint32_t tile_bytes = 0;
    std::vector<Tile> tiles;             // grouped by kernel family, stream order inside a group
    std::vector<Group> groups;
    std::vector<uint32_t> chunk_tiles;   // arrivals each chunk's checksum expects: its tiles, plus one per TRANSPOSE_SPAN
                                         // tile that touches it
    std::vector<uint32_t> inc;           // TRANSPOSE_SPAN tiles: pairs (chunk, ordinal of this arrival among the chunk's),
                                         // a tile's pairs consecutive and ascending by chunk
    std::vector<TensorDev> tdev;
    bool all_unpack_safe = true;
    bool can_accumulate = true;          // every non-empty tensor is contiguous bf16 or f32
    ChunkGeom geom;                      // closed-form geometry of the packed stream
    bool uniform = false;                // the message is one contiguous tensor: geom alone describes the copy
    uint32_t uniform_tensor = 0;         // index of that tensor
    bool all_contig = false;             // every launch group is a contiguous copy (zero pads included)

    uint64_t chunk_padded(uint64_t c) const;
    uint64_t chunk_packed_off(uint64_t c) const { return lane_off[c % k] + (c / k) * B; }
};

// Host-only, allocation-free: the closed-form geometry alone.  Returns an hxt_status.
int make_geom(uint64_t N, uint64_t L, uint64_t B, uint32_t k, uint32_t tile_bytes, ChunkGeom &g);

// Host-only construction of every table (no HIP call).  Returns an hxt_status.
int build_plan(const hxt_tensor_desc_t *tensors, int n_tensors, int n_lanes, size_t chunk_bytes,
               uint32_t tile_bytes, Plan &out);

constexpr uint32_t kDefaultTileBytes = 16384;  // bytes of the stream one workgroup moves (linear kinds)
// A TRANSPOSE tile is at most T x T elements, T chosen so that a tile row is 128-512 bytes.
HXT_HD constexpr uint32_t transpose_tile(uint32_t esize) { return esize <= 2 ? 128u : 64u; }

}  // namespace hxt

#endif
