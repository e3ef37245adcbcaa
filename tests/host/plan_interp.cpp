// Test helper (CPU): executes a plan's work tables one byte at a time, with every
// access bounds-checked and every packed byte's write counted.  It exists to check the
// host planner (tile offsets, clipping at chunk borders, launch groups) before anything
// runs on a GPU; it is compiled together with the planner source only, never with the
// kernels, and is not part of the product.
#include <cstdint>
#include <cstring>
#include <vector>

#include "hxt_internal.h"

using namespace hxt;

namespace {
struct Ctx {
    const Plan &p;
    uint8_t *const *base;
    const uint64_t *storage_bytes;
    uint8_t *packed;
    uint64_t packed_bytes;
    uint8_t *written;   // per packed byte: times written
    int error = 0;
    bool user_ok(uint32_t t, uint64_t off, uint64_t n) { return off + n <= storage_bytes[t]; }
    bool packed_ok(uint64_t off, uint64_t n) { return off + n <= packed_bytes; }
};

uint64_t logical_to_storage(const TensorDev &td, uint64_t byte)
{
    uint64_t e = byte / td.esize, b = byte % td.esize, off = 0;
    for (int d = td.ndim - 1; d >= 0; --d) {
        off += (e % uint64_t(td.shape[d])) * uint64_t(td.stride_b[d]);
        e /= uint64_t(td.shape[d]);
    }
    return off + b;
}

// The per-element kernel's 32-bit address arithmetic, restated for the host: coordinates of the tile's
// first element, plus the element's number carried from the last dim upwards with the plan's
// multiply-shift divisors.  Returns false if any intermediate leaves the range the divisors are exact for.
bool carried_offset(const TensorDev &td, uint64_t e0, uint32_t el, uint64_t *off_out)
{
    uint32_t base[HXT_MAX_DIMS] = {0};
    uint64_t idx = e0;
    for (int d = td.ndim - 1; d >= 0; --d) {
        base[d] = uint32_t(idx % uint64_t(td.shape[d]));
        idx /= uint64_t(td.shape[d]);
    }
    uint64_t x = el, off = 0;
    for (int d = td.ndim - 1; d >= 0; --d) {
        x += base[d];
        if (x >= (uint64_t(1) << 31)) return false;
        if (d > 0) {
            const uint32_t q = fast_div(uint32_t(x), td.dim_div[d]);
            off += uint64_t(uint32_t(x) - q * uint32_t(td.shape[d])) * uint64_t(td.stride_b[d]);
            x = q;
        } else {
            off += x * uint64_t(td.stride_b[0]);
        }
    }
    *off_out = off;
    return true;
}
}  // namespace

// direction 0: pack (user -> packed) from the tables, 1: unpack (packed -> user) from the tables,
// 2: pack from the tables and then, if the message is uniform, again from the closed form.  Returns 0, or a
// negative code: -1 plan error, -2 user access out of bounds, -3 packed access out of
// bounds, -4 tile crosses its chunk, -5 bad group bookkeeping, -6 bad closed-form geometry, -7 the 32-bit
// carried address arithmetic of the per-element kernel disagrees with the plain one, -8 a linear tile's
// recorded offset inside its chunk is wrong.
extern "C" int plan_interp(const hxt_tensor_desc_t *descs, int n_tensors, int n_lanes, uint64_t chunk_bytes,
                           uint32_t tile_bytes, uint8_t *const *base, const uint64_t *storage_bytes,
                           uint8_t *packed, uint64_t packed_bytes, uint8_t *written, int direction,
                           int32_t *kinds_out, int32_t *uniform_out)
{
    Plan p;
    if (build_plan(descs, n_tensors, n_lanes, chunk_bytes, tile_bytes, p) != HXT_OK) return -1;
    if (p.C * p.B != packed_bytes) return -1;
    for (int t = 0; t < n_tensors; ++t) kinds_out[t] = p.tensors[t].kind;
    Ctx c{p, base, storage_bytes, packed, packed_bytes, written};
    uint64_t next = 0;
    for (const Group &g : p.groups) {
        if (g.first != next || g.n_tensors > uint32_t(kMaxGroupTensors)) return -5;
        next = g.first + g.count;
        for (uint32_t i = 0; i < g.count; ++i) {
            const Tile &t = p.tiles[g.first + i];
            const uint32_t ta = g.tensor_base + t.tensor;
            if (t.tensor >= g.n_tensors || ta >= uint32_t(n_tensors)) return -5;
            const TensorDev &td = p.tdev[ta];
            const bool span = t.kind == K_TRANSPOSE_SPAN;      // its rows name their chunks one by one (below)
            uint64_t c_lo = span ? 0 : p.chunk_packed_off(t.chunk), c_hi = span ? 0 : c_lo + p.chunk_padded(t.chunk);
            auto put = [&](uint64_t poff, uint64_t uoff, bool zero) -> int {
                if (!c.packed_ok(poff, 1)) return -3;
                if (poff < c_lo || poff >= c_hi) return -4;
                if (!zero && !c.user_ok(ta, uoff, 1)) return -2;
                if (direction != 1) {
                    packed[poff] = zero ? 0 : base[ta][uoff];
                    if (written[poff] < 255) ++written[poff];
                } else if (!zero) {
                    base[ta][uoff] = packed[poff];
                    if (written[poff] < 255) ++written[poff];
                } else if (written[poff] < 255) {
                    ++written[poff];
                }
                return 0;
            };
            int rc = 0;
            // linear tiles record where they start inside their chunk (the fused tag kernels weigh words by it)
            if (t.kind != K_TRANSPOSE && !span && t.a != t.packed_off - c_lo) return -8;
            // the per-element kernel's carried arithmetic must hold for every linear tile, whichever kernel ends up serving it
            if ((t.kind == K_CONTIG || t.kind == K_ROWS || t.kind == K_ROWS_SPLIT || t.kind == K_GENERIC) && td.all_div) {
                if (t.src_off % td.esize || t.n0 % td.esize) return -7;
                for (uint32_t el = 0; el < t.n0 / td.esize; ++el) {
                    uint64_t off = 0;
                    if (!carried_offset(td, t.src_off / td.esize, el, &off)) return -7;
                    if (off != logical_to_storage(td, t.src_off + uint64_t(el) * td.esize)) return -7;
                }
            }
            switch (t.kind) {
            case K_CONTIG:
                if (g.kernel != K_CONTIG) return -5;
                for (uint64_t b = 0; b < t.n0 && !rc; ++b) rc = put(t.packed_off + b, t.src_off + b, false);
                break;
            case K_ZERO:
                if (g.kernel != K_CONTIG) return -5;
                for (uint64_t b = 0; b < t.n0 && !rc; ++b) rc = put(t.packed_off + b, 0, true);
                break;
            case K_ROWS:
            case K_ROWS_SPLIT:
            case K_GENERIC:
                if (g.kernel != t.kind) return -5;
                if (t.kind == K_ROWS && (t.n0 % 16 || td.row_bytes % 16)) return -5;
                if (t.kind == K_ROWS_SPLIT && (td.row_bytes < 16 || t.src_off % 16)) return -5;
                for (uint64_t b = 0; b < t.n0 && !rc; ++b)
                    rc = put(t.packed_off + b, logical_to_storage(td, t.src_off + b), false);
                break;
            case K_TRANSPOSE:
                if (g.kernel != K_TRANSPOSE || t.n0 > transpose_tile(td.esize) || t.n1 > transpose_tile(td.esize)) return -5;
                if (t.estep < uint32_t(td.esize) || t.estep % uint32_t(td.esize) || t.estep > 16) return -5;
                for (uint64_t i2 = 0; i2 < t.n0 && !rc; ++i2)
                    for (uint64_t j = 0; j < t.n1 && !rc; ++j)
                        for (uint64_t b = 0; b < uint64_t(td.esize) && !rc; ++b)
                            rc = put(t.packed_off + i2 * t.b + j * td.esize + b,
                                     t.src_off + j * t.a + i2 * t.estep + b, false);
                break;
            case K_TRANSPOSE_SPAN: {
                if (g.kernel != K_TRANSPOSE_SPAN || t.n0 > transpose_tile(td.esize) || t.n1 > transpose_tile(td.esize)) return -5;
                if (t.estep < uint32_t(td.esize) || t.estep % uint32_t(td.esize) || t.estep > 16) return -5;
                if (p.B < 1024 || t.ordinal == 0 || uint64_t(t.chunk) + t.ordinal > p.inc.size() / 2) return -5;
                const uint32_t *my = p.inc.data() + 2 * size_t(t.chunk);
                std::vector<uint8_t> touched(t.ordinal, 0);
                for (uint32_t e = 1; e < t.ordinal; ++e)
                    if (my[2 * e] <= my[2 * (e - 1)]) return -5;                    // ascending, each chunk once
                for (uint64_t i2 = 0; i2 < t.n0 && !rc; ++i2)
                    for (uint64_t j = 0; j < t.n1 && !rc; ++j)
                        for (uint64_t b = 0; b < uint64_t(td.esize) && !rc; ++b) {
                            const uint64_t s = t.packed_off + i2 * t.b + j * td.esize + b;   // byte of the logical stream
                            const uint64_t ch = s / p.B;
                            if (ch >= p.C) return -3;
                            uint32_t e = 0;
                            while (e < t.ordinal && my[2 * e] != ch) ++e;
                            if (e == t.ordinal) return -5;                          // a chunk the tile does not announce
                            touched[e] = 1;
                            c_lo = p.chunk_packed_off(ch), c_hi = c_lo + p.chunk_padded(ch);
                            rc = put(c_lo + (s - ch * p.B), t.src_off + j * t.a + i2 * t.estep + b, false);
                        }
                for (uint8_t x : touched)
                    if (!x) return -5;                                              // an arrival announced for nothing
                break;
            }
            default: return -5;
            }
            if (rc) return rc;
        }
    }
    if (next != p.tiles.size()) return -5;
    // per-chunk tile counts (the checksum's "last arrival" test depends on them)
    std::vector<uint32_t> count(p.C, 0);
    std::vector<std::vector<uint8_t>> ord(p.C);
    for (uint64_t ch = 0; ch < p.C; ++ch) ord[ch].assign(p.chunk_tiles[ch], 0);
    for (const Tile &t : p.tiles) {
        if (t.kind == K_TRANSPOSE_SPAN) {                   // one arrival per chunk touched, numbered in the table
            for (uint32_t e = 0; e < t.ordinal; ++e) {
                const uint32_t ch = p.inc[2 * (size_t(t.chunk) + e)], o = p.inc[2 * (size_t(t.chunk) + e) + 1];
                if (ch >= p.C) return -5;
                ++count[ch];
                if (o >= p.chunk_tiles[ch] || ord[ch][o]++) return -5;
            }
            continue;
        }
        ++count[t.chunk];
        if (t.ordinal >= p.chunk_tiles[t.chunk] || ord[t.chunk][t.ordinal]++) return -5;   // ordinals are a permutation
    }
    if (count != p.chunk_tiles) return -5;
    // closed-form geometry: its tiles must cover every chunk's padded bytes exactly once, report
    // the right chunk and the right number of tiles per chunk
    std::vector<uint8_t> seen(packed_bytes, 0);
    std::vector<uint32_t> per_chunk(p.C, 0);
    for (uint32_t i = 0; i < p.geom.ntiles; ++i) {
        const TileSpan t = locate_tile(p.geom, i);
        if (t.chunk >= p.C) return -6;
        const uint64_t c_lo = p.chunk_packed_off(t.chunk), c_hi = c_lo + p.chunk_padded(t.chunk);
        if (t.packed_off < c_lo || t.packed_off + t.len > c_hi || t.len % 256 || t.len == 0) return -6;
        if (t.packed_off - c_lo != t.stream_off - uint64_t(t.chunk) * p.B) return -6;
        if (t.ordinal != per_chunk[t.chunk]) return -6;
        ++per_chunk[t.chunk];
        for (uint64_t b = 0; b < t.len; ++b) ++seen[t.packed_off + b];
    }
    for (uint64_t ch = 0; ch < p.C; ++ch) {
        for (uint64_t b = 0; b < p.chunk_padded(ch); ++b)
            if (seen[p.chunk_packed_off(ch) + b] != 1) return -6;
        const TileSpan any = locate_tile(p.geom, uint32_t(ch) * p.geom.tpc);
        if (any.expected != per_chunk[ch] || any.chunk != ch) return -6;
    }
    if ((p.C == 0) != (p.geom.ntiles == 0)) return -6;
    *uniform_out = p.uniform ? 1 : 0;
    if (p.uniform && direction == 2) {
        // the uniform copy, byte by byte: tensor bytes then zero pad, from the closed form alone
        const uint32_t ta = p.uniform_tensor;
        for (uint32_t i = 0; i < p.geom.ntiles; ++i) {
            const TileSpan t = locate_tile(p.geom, i);
            for (uint64_t b = 0; b < t.len; ++b) {
                const uint64_t s = t.stream_off + b;
                if (s < p.geom.N) {
                    if (!c.user_ok(ta, s, 1)) return -2;
                    packed[t.packed_off + b] = base[ta][s];
                } else {
                    packed[t.packed_off + b] = 0;
                }
            }
        }
    }
    return 0;
}

// Exhaustive check of the multiply-shift division used by the row-gather kernel.
extern "C" int fastdiv_check(uint32_t d, const uint32_t *ns, int count)
{
    FastDiv f = make_fastdiv(d);
    for (int i = 0; i < count; ++i) {
        uint32_t q = uint32_t((uint64_t(ns[i]) * f.mul) >> (31 + f.shift));
        if (q != ns[i] / d) return -1;
    }
    return 0;
}
