// Host planner of libhxt: geometry of the stream, chunk/lane layout and the
// per-workgroup work tables.  Pure C++, no HIP: it is the "control plane on the
// host" half of the paper's Section 2.2 mechanism; the data plane (kernels)
// only follows the tables built here.
#include "hxt_internal.h"

#include <algorithm>
#include <cstring>

namespace hxt {

static inline uint64_t roundup(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

FastDiv make_fastdiv(uint32_t d)
{
    // s = ceil(log2 d); mul = floor(2^(31+s) / d) + 1 fits 32 bits and makes
    // (n * mul) >> (31 + s) == n / d for every n < 2^31 (error term e = mul*d - 2^(31+s)
    // satisfies 0 < e <= 2^s, so n*e < 2^(31+s)).
    uint32_t s = 0;
    while ((uint64_t(1) << s) < d) ++s;
    uint64_t mul = (uint64_t(1) << (31 + s)) / d + 1;
    return FastDiv{uint32_t(mul), s};
}

// Closed-form geometry of a packed stream of L bytes (a multiple of 256) cut into chunks of B bytes over k
// lanes, with tiles of tile_bytes; N = tensor bytes when the stream is one contiguous tensor, else 0.
int make_geom(uint64_t N, uint64_t L, uint64_t B, uint32_t k, uint32_t tile_bytes, ChunkGeom &g)
{
    std::memset(&g, 0, sizeof g);
    const uint64_t C = (L + B - 1) / B;
    if (C >= (uint64_t(1) << 31)) return HXT_EUNSUPPORTED;
    g.N = N;
    g.L = L;
    g.B = B;
    g.k = k;
    g.C = uint32_t(C);
    g.tile = tile_bytes;
    const uint64_t tpc = (B + tile_bytes - 1) / tile_bytes;
    if (tpc * std::max<uint64_t>(C, 1) >= (uint64_t(1) << 31)) return HXT_EUNSUPPORTED;
    g.tpc = uint32_t(tpc);
    g.q = uint32_t(C / k);
    g.r = uint32_t(C % k);
    const uint64_t last = C ? L - (C - 1) * B : 0;
    g.last_tiles = uint32_t((last + tile_bytes - 1) / tile_bytes);
    g.ntiles = C ? uint32_t((C - 1) * tpc) + g.last_tiles : 0;
    g.div_tpc = make_fastdiv(g.tpc);
    g.div_k = make_fastdiv(g.k);
    return HXT_OK;
}

static int dtype_size(hxt_dtype_t dt)
{
    switch (dt) {
    case HXT_U8: return 1;
    case HXT_F16: return 2;
    case HXT_BF16: return 2;
    case HXT_F32: return 4;
    case HXT_F64: return 8;
    }
    return 0;
}

uint64_t Plan::chunk_padded(uint64_t c) const
{
    uint64_t lo = c * B, hi = std::min((c + 1) * B, L);
    return hi > lo ? hi - lo : 0;
}

// Drop extent-1 dims and merge neighbours that are contiguous with each other
// (stride[d] == shape[d+1] * stride[d+1]); the logical order of elements is unchanged.
static void merge_dims(const hxt_tensor_desc_t &in, TensorPlan &t)
{
    int64_t shp[HXT_MAX_DIMS], str[HXT_MAX_DIMS];
    int n = 0;
    int64_t run = 1;
    for (int d = in.ndim - 1; d >= 0; --d) {           // contiguous strides when none are given
        int64_t s = in.strides ? in.strides[d] : run;
        run *= std::max<int64_t>(in.shape[d], 1);
        if (in.shape[d] == 1) continue;
        shp[n] = in.shape[d];
        str[n] = s;
        ++n;
    }
    std::reverse(shp, shp + n);
    std::reverse(str, str + n);
    int m = 0;
    for (int d = 0; d < n; ++d) {
        if (m > 0 && t.stride[m - 1] == shp[d] * str[d]) {
            t.shape[m - 1] *= shp[d];
            t.stride[m - 1] = str[d];
        } else {
            t.shape[m] = shp[d];
            t.stride[m] = str[d];
            ++m;
        }
    }
    t.ndim = m;
}

// A view is safe to write through when no two index tuples share an address.  Sufficient
// test: with dims sorted by stride, each stride exceeds the largest offset the smaller
// dims can reach.  Views that fail it (stride 0, interleavings) are treated as aliasing.
static bool view_is_injective(const TensorPlan &t)
{
    int idx[HXT_MAX_DIMS];
    for (int d = 0; d < t.ndim; ++d) idx[d] = d;
    std::sort(idx, idx + t.ndim, [&](int a, int b) { return t.stride[a] < t.stride[b]; });
    uint64_t reach = 0;                                  // largest offset the dims seen so far can produce
    for (int j = 0; j < t.ndim; ++j) {
        int d = idx[j];
        if (uint64_t(t.stride[d]) <= reach) return false;   // also rejects stride 0 (reach starts at 0)
        reach += uint64_t(t.shape[d] - 1) * uint64_t(t.stride[d]);
    }
    return true;
}

static Kind classify(const TensorPlan &t, uint64_t chunk_bytes)
{
    if (t.elems == 0) return K_NONE;
    if (t.ndim == 0) return K_CONTIG;                               // one element
    const int last = t.ndim - 1;
    if (t.stride[last] == 1) {
        if (t.ndim == 1) return K_CONTIG;
        uint64_t row_bytes = uint64_t(t.shape[last]) * t.esize;
        uint64_t rows = t.elems / uint64_t(t.shape[last]);
        bool ok = row_bytes % 16 == 0 && row_bytes < (1u << 30) && rows < (1u << 31);
        for (int d = 0; d < last; ++d)
            ok = ok && (uint64_t(t.stride[d]) * t.esize) % 16 == 0 && t.shape[d] < (int64_t(1) << 31);
        if (ok) return K_ROWS;
        // runs or pitches that are not multiples of 16 bytes: still a gather of runs, with the tensor side
        // accessed in narrower pieces, as long as a 16-byte vector meets at most one run boundary
        bool split = row_bytes >= 16 && row_bytes < (1u << 30) && rows < (1u << 31);
        for (int d = 0; d < last; ++d) split = split && t.shape[d] < (int64_t(1) << 31);
        return split ? K_ROWS_SPLIT : K_GENERIC;
    }
    // The dim before the last runs along the storage (stride one, or a few elements: at most 16 bytes, so that
    // neighbouring elements still share memory bursts) and the last dim jumps further: a transpose through LDS.
    // Tiles stay inside one chunk when a chunk holds at least a tile's height of rows of the packed side, so that
    // all but the tiles at chunk borders are full; flatter chunks get tiles that span chunks (chunks of at least
    // 1 KiB, so that a tile row meets at most one chunk border).
    const bool classic = t.ndim >= 2 && t.stride[last] > 1 && t.stride[last - 1] == 1;
    const bool strided = t.ndim >= 2 && t.stride[last - 1] > 1 && t.stride[last] > t.stride[last - 1] &&
                         uint64_t(t.stride[last - 1]) * t.esize <= 16;
    if (classic || strided) {
        const bool tall = uint64_t(t.shape[last]) * t.esize * transpose_tile(uint32_t(t.esize)) <= chunk_bytes;
        if (tall) return K_TRANSPOSE;
        if (chunk_bytes >= 1024) return K_TRANSPOSE_SPAN;
        if (classic) return K_TRANSPOSE;
    }
    return K_GENERIC;
}

static TensorDev make_tensor_dev(const TensorPlan &t)
{
    TensorDev d;
    std::memset(&d, 0, sizeof d);
    d.ndim = t.ndim;
    d.esize = t.esize;
    for (int i = 0; i < t.ndim; ++i) {
        d.shape[i] = t.shape[i];
        d.stride_b[i] = t.stride[i] * t.esize;
    }
    if (t.kind == K_ROWS || t.kind == K_ROWS_SPLIT) {
        d.row_bytes = uint32_t(t.shape[t.ndim - 1] * t.esize);
        d.low_or = d.row_bytes;
        for (int i = 0; i < t.ndim - 1; ++i) d.low_or |= uint32_t(uint64_t(d.stride_b[i]) & 0xFFu);
        d.row_div = make_fastdiv(d.row_bytes);
        for (int i = 0; i < t.ndim - 1; ++i) d.dim_div[i] = make_fastdiv(uint32_t(t.shape[i]));
    }
    // For the per-element kernel: all_div says that dim_div is valid for every dim, with room for a carry.
    bool small = t.ndim > 0;
    for (int i = 0; i < t.ndim; ++i) small = small && t.shape[i] >= 1 && t.shape[i] <= (int64_t(1) << 30);
    d.all_div = small ? 1u : 0u;
    if (small)
        for (int i = 0; i < t.ndim; ++i) d.dim_div[i] = make_fastdiv(uint32_t(t.shape[i]));
    return d;
}

namespace {
struct RawTile {
    Tile t;
    uint32_t tensor_abs;
};

struct Builder {
    Plan &p;
    std::vector<RawTile> by_kernel[8];   // indexed by kernel kind (1..4, 6 and 7)
    explicit Builder(Plan &plan) : p(plan) {}

    void add(Kind kernel, Kind kind, uint32_t tensor, uint64_t packed_off, uint64_t src_off, uint64_t a,
             uint64_t b, uint32_t chunk, uint32_t n0, uint32_t n1, uint32_t estep = 0)
    {
        RawTile r;
        r.t = Tile{packed_off, src_off, a, b, chunk, 0, uint32_t(kind), n0, n1, 0, estep, 0};
        r.tensor_abs = tensor;
        by_kernel[kernel].push_back(r);
    }

    // Cut stream bytes [s0, s1) of tensor ti (tensor-relative start lo0) at chunk and tile
    // boundaries and emit linear tiles of the given kind.
    void linear(Kind kernel, Kind kind, uint32_t ti, uint64_t s0, uint64_t s1, uint64_t lo0, uint32_t step)
    {
        uint64_t s = s0;
        while (s < s1) {
            uint64_t c = s / p.B;
            uint64_t end = std::min({(c + 1) * p.B, s1, s + step});
            add(kernel, kind, ti, p.chunk_packed_off(c) + (s - c * p.B), lo0 + (s - s0), s - c * p.B, 0, uint32_t(c),
                uint32_t(end - s), 0);
            s = end;
        }
    }

    void transpose(uint32_t ti)
    {
        const TensorPlan &t = p.tensors[ti];
        const int n = t.ndim;
        const uint64_t e = t.esize, I = t.shape[n - 2], J = t.shape[n - 1], sI = t.stride[n - 2], sJ = t.stride[n - 1];
        const uint64_t T = transpose_tile(uint32_t(e));
        auto batch_off = [&](uint64_t batch) {           // storage offset (elements) of a batch index
            uint64_t off = 0;
            for (int d = n - 3; d >= 0; --d) {
                off += (batch % uint64_t(t.shape[d])) * uint64_t(t.stride[d]);
                batch /= uint64_t(t.shape[d]);
            }
            return off;
        };
        auto region = [&](uint64_t c, uint64_t r_lo, uint64_t r_hi, uint64_t c_lo, uint64_t c_hi) {
            uint64_t rr = r_lo;
            while (rr < r_hi) {
                uint64_t batch = rr / I, i0 = rr % I;
                uint64_t ni = std::min({r_hi - rr, I - i0, T});
                for (uint64_t cc = c_lo; cc < c_hi; cc += T) {
                    uint64_t nj = std::min(T, c_hi - cc);
                    uint64_t stream = t.stream_off + (rr * J + cc) * e;
                    add(K_TRANSPOSE, K_TRANSPOSE, ti, p.chunk_packed_off(c) + (stream - c * p.B),
                        (batch_off(batch) + i0 * sI + cc * sJ) * e, sJ * e, J * e, uint32_t(c), uint32_t(ni), uint32_t(nj),
                        uint32_t(sI * e));
                }
                rr += ni;
            }
        };
        uint64_t s = t.stream_off, s_end = t.stream_off + t.bytes;
        while (s < s_end) {
            uint64_t c = s / p.B;
            uint64_t end = std::min((c + 1) * p.B, s_end);
            uint64_t ea = (s - t.stream_off) / e, eb = (end - t.stream_off) / e;
            uint64_t r0 = ea / J, c0 = ea % J, r1 = eb / J, c1 = eb % J;
            if (r0 == r1) {
                region(c, r0, r0 + 1, c0, c1);
            } else {
                if (c0 != 0) {
                    region(c, r0, r0 + 1, c0, J);
                    ++r0;
                }
                if (r1 > r0) region(c, r0, r1, 0, J);
                if (c1 != 0) region(c, r1, r1 + 1, 0, c1);
            }
            s = end;
        }
    }

    // The same blocks of the logical matrix without regard to chunks: every tile is a full T x T block (clipped by
    // the matrix only).  A tile's entries in p.inc name the chunks its rows lie in; their ordinals are set once
    // all tiles are known.
    void transpose_span(uint32_t ti)
    {
        const TensorPlan &t = p.tensors[ti];
        const int n = t.ndim;
        const uint64_t e = t.esize, I = t.shape[n - 2], J = t.shape[n - 1], sI = t.stride[n - 2], sJ = t.stride[n - 1];
        const uint64_t T = transpose_tile(uint32_t(e)), batches = t.elems / (I * J);
        for (uint64_t batch = 0; batch < batches; ++batch) {
            uint64_t boff = 0, rest = batch;             // storage offset (elements) of the batch index
            for (int d = n - 3; d >= 0; --d) {
                boff += (rest % uint64_t(t.shape[d])) * uint64_t(t.stride[d]);
                rest /= uint64_t(t.shape[d]);
            }
            for (uint64_t i0 = 0; i0 < I; i0 += T) {
                const uint64_t ni = std::min(T, I - i0);
                for (uint64_t j0 = 0; j0 < J; j0 += T) {
                    const uint64_t nj = std::min(T, J - j0);
                    const uint64_t s0 = t.stream_off + ((batch * I + i0) * J + j0) * e;
                    const size_t first = p.inc.size() / 2;
                    uint64_t last_c = ~uint64_t(0);
                    for (uint64_t i = 0; i < ni; ++i) {
                        const uint64_t s = s0 + i * J * e;
                        for (uint64_t c : {s / p.B, (s + nj * e - 1) / p.B})
                            if (c != last_c) {
                                p.inc.push_back(uint32_t(c));
                                p.inc.push_back(0);
                                last_c = c;
                            }
                    }
                    add(K_TRANSPOSE_SPAN, K_TRANSPOSE_SPAN, ti, s0, (boff + i0 * sI + j0 * sJ) * e, sJ * e, J * e,
                        uint32_t(first), uint32_t(ni), uint32_t(nj), uint32_t(sI * e));
                    by_kernel[K_TRANSPOSE_SPAN].back().t.ordinal = uint32_t(p.inc.size() / 2 - first);
                }
            }
        }
    }
};
}  // namespace

int build_plan(const hxt_tensor_desc_t *descs, int n_tensors, int n_lanes, size_t chunk_bytes,
               uint32_t tile_bytes, Plan &p)
{
    if (n_tensors < 0 || (n_tensors > 0 && !descs)) return HXT_EINVAL;
    if (n_lanes < 1 || n_lanes > 1024) return HXT_EINVAL;
    if (chunk_bytes == 0 || chunk_bytes % HXT_ALIGN) return HXT_EINVAL;
    if (tile_bytes == 0 || tile_bytes % HXT_ALIGN || tile_bytes > (1u << 24)) return HXT_EINVAL;
    const uint64_t kMaxBytes = uint64_t(1) << 40;

    p.B = chunk_bytes;
    p.k = n_lanes;
    p.tile_bytes = tile_bytes;
    p.tensors.resize(n_tensors);
    uint64_t off = 0;
    for (int i = 0; i < n_tensors; ++i) {
        const hxt_tensor_desc_t &d = descs[i];
        TensorPlan &t = p.tensors[i];
        if (d.ndim < 0 || d.ndim > HXT_MAX_DIMS || (d.ndim > 0 && !d.shape)) return HXT_EINVAL;
        t.esize = dtype_size(d.dtype);
        if (t.esize == 0) return HXT_EINVAL;
        t.dtype = d.dtype;
        uint64_t elems = 1;
        for (int k = 0; k < d.ndim; ++k) {
            if (d.shape[k] < 0 || (d.strides && d.strides[k] < 0)) return HXT_EINVAL;
            if (d.shape[k] != 0 && elems > kMaxBytes / uint64_t(d.shape[k])) return HXT_EUNSUPPORTED;
            elems *= uint64_t(d.shape[k]);
        }
        if (elems * t.esize > kMaxBytes) return HXT_EUNSUPPORTED;
        if (d.strides && elems > 0) {                    // the view must stay addressable: its farthest byte below 2^62
            unsigned __int128 reach = 0;
            for (int k = 0; k < d.ndim; ++k)
                reach += (unsigned __int128)(uint64_t(d.shape[k]) - 1) * uint64_t(d.strides[k]);
            if ((reach + 1) * unsigned(t.esize) > ((unsigned __int128)1 << 62)) return HXT_EUNSUPPORTED;
        }
        t.elems = elems;
        t.bytes = elems * t.esize;
        t.stream_off = off;
        if (elems > 0) merge_dims(d, t);
        t.kind = classify(t, chunk_bytes);
        t.unpack_safe = elems == 0 || view_is_injective(t);
        p.all_unpack_safe = p.all_unpack_safe && t.unpack_safe;
        if (elems > 0 && !(t.kind == K_CONTIG && (t.dtype == HXT_BF16 || t.dtype == HXT_F32))) p.can_accumulate = false;
        p.N += t.bytes;
        off = roundup(off + t.bytes, HXT_ALIGN);
        if (off > kMaxBytes) return HXT_EUNSUPPORTED;
    }
    p.L = off;
    p.C = (p.L + p.B - 1) / p.B;
    if (p.C >= (uint64_t(1) << 31)) return HXT_EUNSUPPORTED;

    // lanes: round-robin deal; lane l gets C/k chunks plus one if l < C mod k
    p.lane_off.assign(p.k + 1, 0);
    p.lane_chunks.assign(p.k, 0);
    for (int l = 0; l < p.k; ++l) {
        p.lane_chunks[l] = p.C / p.k + (uint64_t(l) < p.C % p.k ? 1 : 0);
        p.lane_off[l + 1] = p.lane_off[l] + p.lane_chunks[l] * p.B;
    }

    // work tables
    Builder b(p);
    p.tdev.resize(n_tensors);
    for (int i = 0; i < n_tensors; ++i) {
        const TensorPlan &t = p.tensors[i];
        p.tdev[i] = make_tensor_dev(t);
        if (t.bytes == 0) continue;
        const uint64_t data_end = t.stream_off + t.bytes, ext_end = roundup(data_end, HXT_ALIGN);
        switch (t.kind) {
        case K_CONTIG: b.linear(K_CONTIG, K_CONTIG, i, t.stream_off, data_end, 0, tile_bytes); break;
        case K_ROWS: b.linear(K_ROWS, K_ROWS, i, t.stream_off, data_end, 0, tile_bytes); break;
        case K_ROWS_SPLIT: b.linear(K_ROWS_SPLIT, K_ROWS_SPLIT, i, t.stream_off, data_end, 0, tile_bytes); break;
        case K_GENERIC: b.linear(K_GENERIC, K_GENERIC, i, t.stream_off, data_end, 0, tile_bytes); break;
        case K_TRANSPOSE: b.transpose(i); break;
        case K_TRANSPOSE_SPAN: b.transpose_span(i); break;
        default: break;
        }
        if (ext_end > data_end) b.linear(K_CONTIG, K_ZERO, i, data_end, ext_end, t.bytes, HXT_ALIGN);
    }
    uint64_t total = 0;
    for (auto &v : b.by_kernel) total += v.size();
    if (total >= (uint64_t(1) << 31)) return HXT_EUNSUPPORTED;
    p.tiles.reserve(total);
    p.chunk_tiles.assign(p.C, 0);
    if (p.inc.size() / 2 >= (uint64_t(1) << 31)) return HXT_EUNSUPPORTED;
    for (Kind kern : {K_CONTIG, K_ROWS, K_ROWS_SPLIT, K_TRANSPOSE, K_GENERIC, K_TRANSPOSE_SPAN}) {
        auto &v = b.by_kernel[kern];
        size_t i = 0;
        while (i < v.size()) {
            Group g{kern, uint32_t(p.tiles.size()), 0, v[i].tensor_abs, 0};
            while (i < v.size() && v[i].tensor_abs < g.tensor_base + kMaxGroupTensors) {
                Tile t = v[i].t;
                t.tensor = v[i].tensor_abs - g.tensor_base;
                g.n_tensors = std::max(g.n_tensors, t.tensor + 1);
                if (kern == K_TRANSPOSE_SPAN) {              // one arrival at every chunk the tile touches
                    for (uint32_t e = 0; e < t.ordinal; ++e) {
                        const size_t at = 2 * (size_t(t.chunk) + e);
                        p.inc[at + 1] = p.chunk_tiles[p.inc[at]]++;
                    }
                } else {
                    t.ordinal = p.chunk_tiles[t.chunk]++;
                }
                p.tiles.push_back(t);
                ++g.count;
                ++i;
            }
            p.groups.push_back(g);
        }
    }
    // closed-form geometry of the packed stream (stand-alone checksum; uniform copy)
    ChunkGeom &g = p.geom;
    if (int rc = make_geom(0, p.L, p.B, uint32_t(p.k), tile_bytes, g); rc != HXT_OK) return rc;
    int live = 0;
    for (int i = 0; i < n_tensors; ++i)
        if (p.tensors[i].bytes) {
            ++live;
            p.uniform_tensor = uint32_t(i);
        }
    p.uniform = live == 1 && p.tensors[p.uniform_tensor].kind == K_CONTIG;
    p.all_contig = true;
    for (const Group &gr : p.groups) p.all_contig = p.all_contig && gr.kernel == K_CONTIG;
    g.N = p.uniform ? p.tensors[p.uniform_tensor].bytes : 0;
    return HXT_OK;
}

}  // namespace hxt
