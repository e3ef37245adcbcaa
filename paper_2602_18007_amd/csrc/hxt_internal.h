// Internal structures shared by the host planner and the HIP kernels of libhxt.
// Not part of the ABI.
#ifndef HXT_INTERNAL_H
#define HXT_INTERNAL_H

#include <cstdint>
#include <vector>

#include "hxt.h"

namespace hxt {

// Which kernel family moves a piece of the stream.
enum Kind : uint16_t {
    K_NONE = 0,
    K_CONTIG = 1,     // tensor bytes are contiguous in memory: straight 128-bit copy
    K_ROWS = 2,       // innermost dimension contiguous, 16-byte friendly rows: gather of runs
    K_TRANSPOSE = 3,  // innermost logical dim strided, second innermost contiguous: LDS tile transpose
    K_GENERIC = 4,    // anything else: one element at a time
    K_ZERO = 5,       // pad bytes between tensors / after the last one (byte granular, < 256 bytes)
    K_CSUM = 6        // stand-alone checksum pass over a packed chunk
};

// One unit of work for one workgroup.  64 bytes of 32/64-bit fields, read with scalar loads.
//   linear kinds (CONTIG, ROWS, GENERIC, ZERO, CSUM):
//     packed_off : first packed byte of the piece (CONTIG/ROWS/GENERIC/CSUM: multiple of 256)
//     src_off    : logical byte offset inside the tensor (equals the storage offset for CONTIG)
//     n0         : bytes of the piece
//   TRANSPOSE (a 2-D block of ni logical rows x nj logical columns inside one chunk):
//     packed_off : packed byte of element (i0, j0);  b = packed row pitch in bytes
//     src_off    : storage byte of element (i0, j0); a = storage pitch between columns in bytes
//     n0 = ni (rows, contiguous in storage), n1 = nj (columns, contiguous in the packed stream)
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
    uint32_t reserved[3];
};
static_assert(sizeof(Tile) == 64, "Tile must stay 64 bytes");

// Exact unsigned division of n < 2^31 by a fixed d < 2^31: q = (n * mul) >> (31 + shift).
struct FastDiv {
    uint32_t mul;
    uint32_t shift;
};
FastDiv make_fastdiv(uint32_t d);

// Per-tensor view description for the ROWS and GENERIC kernels (merged dims, logical order).
struct TensorDev {
    int32_t ndim;                      // merged dims; for ROWS the last one is the contiguous run
    int32_t esize;
    uint32_t row_bytes;                // ROWS: bytes of one contiguous run
    FastDiv row_div;                   // ROWS: division by row_bytes
    FastDiv dim_div[HXT_MAX_DIMS];     // ROWS: division by shape[d] for the outer dims
    int64_t shape[HXT_MAX_DIMS];
    int64_t stride_b[HXT_MAX_DIMS];    // bytes
};

constexpr int kMaxGroupTensors = 64;   // base pointers passed by value per launch

struct TensorPlan {
    int ndim = 0;                      // merged
    int64_t shape[HXT_MAX_DIMS] = {0};
    int64_t stride[HXT_MAX_DIMS] = {0};  // elements
    int esize = 1;
    uint64_t elems = 0, bytes = 0, stream_off = 0;
    Kind kind = K_NONE;
    bool unpack_safe = true;
};

struct Group {          // one kernel launch
    Kind kernel;        // K_CONTIG (serves ZERO tiles too), K_ROWS, K_TRANSPOSE, K_GENERIC
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
    std::vector<Tile> tiles;             // pack/unpack groups first, then the CSUM tiles
    std::vector<Group> groups;
    uint32_t csum_first = 0, csum_count = 0;
    std::vector<TensorDev> tdev;
    bool all_unpack_safe = true;

    // device copies (owned)
    Tile *d_tiles = nullptr;
    TensorDev *d_tensors = nullptr;
    int device = -1;

    uint64_t chunk_padded(uint64_t c) const;
    uint64_t chunk_packed_off(uint64_t c) const { return lane_off[c % k] + (c / k) * B; }
};

// Host-only construction of every table (no HIP call).  Returns an hxt_status.
int build_plan(const hxt_tensor_desc_t *tensors, int n_tensors, int n_lanes, size_t chunk_bytes,
               uint32_t tile_bytes, Plan &out);

constexpr uint32_t kDefaultTileBytes = 16384;  // bytes of the stream one workgroup moves (linear kinds)
constexpr uint32_t kTransposeTile = 64;        // a TRANSPOSE tile is at most 64 x 64 elements

}  // namespace hxt

struct hxt_plan {
    hxt::Plan p;
};

#endif
