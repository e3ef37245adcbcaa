/*
 * hxt_oracle.c -- slow, plain CPU statement of what the pipeline-parallel
 * boundary transfer computes.  TEST INFRASTRUCTURE ONLY: nothing in the
 * product library includes, links or calls this file, and this file includes
 * nothing of the product (it restates every constant it needs).
 *
 * What it models (paper, Section 2.2, "CPU-offloading P2P mechanism"): the
 * sender copies the user tensor device-to-device into a chunk buffer, the
 * chunk buffer is shipped, and the receiver does the symmetric copy back into
 * its own tensor.  Section 2.1 (MPDT) spreads pipeline traffic over several
 * independent NICs ("lanes" here) and describes the CPU-forwarding variant,
 * where the chunk buffer additionally crosses to host memory and back.
 *
 * The paper fixes none of the constants.  The contract implemented here:
 *
 *  1. Logical stream.  Tensors t = 0..T-1 are laid one after another; tensor t
 *     contributes its elements in row-major order of its SHAPE (last index
 *     fastest), element (i_0..i_{n-1}) being read from storage byte
 *     esize * sum_d i_d * stride_d.  Tensor t starts at stream byte off_t with
 *     off_0 = 0 and off_{t+1} = roundup(off_t + bytes_t, 256); the stream ends
 *     at L = roundup(off_{T-1} + bytes_{T-1}, 256).  Bytes between tensors and
 *     after the last one are zero.  N = sum_t bytes_t is the message size.
 *  2. Chunks.  Chunk c is stream bytes [c*B, min((c+1)*B, L)), B = chunk_bytes
 *     (a multiple of 256).  C = ceil(L / B).
 *  3. Lanes.  Chunks are dealt round-robin: lane(c) = c mod k, slot(c) = c div k.
 *  4. Packed buffer.  Lane-major: lane l owns one contiguous region holding its
 *     chunks in slot order, every slot B bytes wide; regions follow each other
 *     in lane order.  Slot bytes past the end of a short last chunk are
 *     unspecified (never written, summed or compared).
 *  5. Staging a lane = copying that lane's used region unchanged.
 *  6. Unpack = the inverse of 1-4 for every tensor byte; pad bytes are dropped.
 *  7. Checksum of chunk c = sum of its little-endian 32-bit words, mod 2^64.
 *  Widenings, each stated where it is defined below: receive-and-accumulate, a second
 *  position-weighted sum per chunk, and a 64-byte tag per chunk (seal / verify).
 *
 * Style: one element at a time, every position recomputed from the formulas
 * above; no chunk table, no dimension merging, no blocking.  The counting
 * loops (chunks per lane, payload per chunk) are deliberately loops.
 *
 * Pins (see tests/test_oracle_pins.py): hand-written chunk orders and sizes in
 * tests/golden/, NumPy's own strided-view flattening as the logical stream,
 * memcpy for the k=1 contiguous case, closed-form checksums, Python big-int
 * sums, round-trip identity, forward map vs inverse map; the accumulate arithmetic in
 * tests/test_oracle_accumulate_pins.py, the chunk tags in tests/test_oracle_tag_pins.py
 * (hand-written record bytes, planted faults).  The end-to-end
 * training throughput and loss results of the paper's Section 3 are not
 * reproduced by anything here: parity unpinned, out of scope.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define HXO_ALIGN 256      /* alignment of tensor starts and of the stream end */
#define HXO_MAXDIM 8

/* A message: T tensors; row t of shape/stride (HXO_MAXDIM wide) has ndim[t] valid entries. */
typedef struct {
    int T;
    const int32_t *ndim;      /* [T] */
    const int64_t *shape;     /* [T][HXO_MAXDIM] */
    const int64_t *stride;    /* [T][HXO_MAXDIM], in elements, >= 0 */
    const int32_t *esize;     /* [T] element size in bytes */
} hxo_msg;

static int64_t roundup(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

/* ---- step 1: sizes of the logical stream ---------------------------------- */

int64_t hxo_tensor_elems(const hxo_msg *m, int t)
{
    int64_t n = 1;
    for (int d = 0; d < m->ndim[t]; ++d) n *= m->shape[t * HXO_MAXDIM + d];
    return n;
}

int64_t hxo_tensor_bytes(const hxo_msg *m, int t)
{
    return hxo_tensor_elems(m, t) * m->esize[t];
}

/* off_t; for t == T this is the stream length L */
int64_t hxo_tensor_offset(const hxo_msg *m, int t)
{
    int64_t off = 0;
    for (int u = 0; u < t; ++u) off = roundup(off + hxo_tensor_bytes(m, u), HXO_ALIGN);
    return off;
}

int64_t hxo_message_bytes(const hxo_msg *m)
{
    int64_t n = 0;
    for (int t = 0; t < m->T; ++t) n += hxo_tensor_bytes(m, t);
    return n;
}

int64_t hxo_stream_bytes(const hxo_msg *m) { return hxo_tensor_offset(m, m->T); }

/* ---- steps 2-4: chunks, lanes, packed layout ------------------------------- */

int64_t hxo_num_chunks(int64_t L, int64_t B) { return (L + B - 1) / B; }

int64_t hxo_chunk_lane(int64_t c, int k) { return c % k; }
int64_t hxo_chunk_slot(int64_t c, int k) { return c / k; }

/* number of chunks dealt to lane l: counted, not derived */
int64_t hxo_lane_chunks(int64_t L, int64_t B, int k, int l)
{
    int64_t n = 0, C = hxo_num_chunks(L, B);
    for (int64_t c = 0; c < C; ++c) if (c % k == l) ++n;
    return n;
}

/* first packed byte of lane l's region; l == k gives packed_bytes */
int64_t hxo_lane_offset(int64_t L, int64_t B, int k, int l)
{
    int64_t off = 0;
    for (int j = 0; j < l; ++j) off += hxo_lane_chunks(L, B, k, j) * B;
    return off;
}

int64_t hxo_packed_bytes(int64_t L, int64_t B, int k) { return hxo_lane_offset(L, B, k, k); }

/* length of chunk c in the stream (short only for the last chunk) */
int64_t hxo_chunk_padded(int64_t L, int64_t B, int64_t c)
{
    int64_t lo = c * B, hi = (c + 1) * B;
    if (hi > L) hi = L;
    return hi > lo ? hi - lo : 0;
}

int64_t hxo_chunk_packed_offset(int64_t L, int64_t B, int k, int64_t c)
{
    return hxo_lane_offset(L, B, k, (int)hxo_chunk_lane(c, k)) + hxo_chunk_slot(c, k) * B;
}

/* used bytes of lane l: up to the last padded byte of its last chunk */
int64_t hxo_lane_used(int64_t L, int64_t B, int k, int l)
{
    int64_t n = hxo_lane_chunks(L, B, k, l);
    if (n == 0) return 0;
    int64_t last = (n - 1) * k + l;              /* the chunk in the lane's last slot */
    return (n - 1) * B + hxo_chunk_padded(L, B, last);
}

/* packed position of stream byte s */
int64_t hxo_stream_to_packed(int64_t L, int64_t B, int k, int64_t s)
{
    int64_t c = s / B;
    return hxo_chunk_packed_offset(L, B, k, c) + (s - c * B);
}

/* real tensor bytes inside chunk c: counted tensor by tensor */
int64_t hxo_chunk_payload(const hxo_msg *m, int64_t B, int64_t c)
{
    int64_t lo = c * B, hi = (c + 1) * B, n = 0;
    for (int t = 0; t < m->T; ++t) {
        int64_t a = hxo_tensor_offset(m, t), b = a + hxo_tensor_bytes(m, t);
        int64_t x = a > lo ? a : lo, y = b < hi ? b : hi;
        if (y > x) n += y - x;
    }
    return n;
}

/* storage byte offset (from the tensor's base pointer) of logical element e */
int64_t hxo_element_storage_offset(const hxo_msg *m, int t, int64_t e)
{
    const int64_t *sh = m->shape + t * HXO_MAXDIM, *st = m->stride + t * HXO_MAXDIM;
    int64_t off = 0;
    for (int d = m->ndim[t] - 1; d >= 0; --d) {     /* last index fastest */
        int64_t i = e % sh[d];
        e /= sh[d];
        off += i * st[d];
    }
    return off * m->esize[t];
}

/* ---- step 2 of the transfer: pack ------------------------------------------ */

/* The k+1 lane offsets do not depend on the element, so pack/unpack evaluate them
 * once per call (through hxo_lane_offset above) instead of once per byte; the
 * per-byte position is still computed from the formulas of steps 2-4. */
typedef struct { int64_t L, B; int k; int64_t lane_off[1025]; } hxo_geom;

static int geom_init(hxo_geom *g, const hxo_msg *m, int64_t B, int k)
{
    if (k < 1 || k > 1024 || B <= 0 || B % HXO_ALIGN) return -1;
    g->L = hxo_stream_bytes(m); g->B = B; g->k = k;
    for (int l = 0; l <= k; ++l) g->lane_off[l] = hxo_lane_offset(g->L, B, k, l);
    return 0;
}

static int64_t geom_map(const hxo_geom *g, int64_t s)
{
    int64_t c = s / g->B;
    return g->lane_off[c % g->k] + (c / g->k) * g->B + (s - c * g->B);
}

/* zero every packed byte that belongs to the stream, then drop the tensor bytes in */
int hxo_pack(const hxo_msg *m, const uint8_t *const *base, int64_t B, int k,
             uint8_t *packed, int nthreads)
{
    hxo_geom g;
    if (geom_init(&g, m, B, k)) return -1;
    (void)nthreads;
#pragma omp parallel for num_threads(nthreads) schedule(static)
    for (int64_t s = 0; s < g.L; s += HXO_ALIGN)
        memset(packed + geom_map(&g, s), 0, HXO_ALIGN);   /* a 256-byte unit never straddles a chunk */
    for (int t = 0; t < m->T; ++t) {
        int64_t off = hxo_tensor_offset(m, t), n = hxo_tensor_elems(m, t);
        int es = m->esize[t];
#pragma omp parallel for num_threads(nthreads) schedule(static)
        for (int64_t e = 0; e < n; ++e) {
            const uint8_t *src = base[t] + hxo_element_storage_offset(m, t, e);
            for (int b = 0; b < es; ++b)
                packed[geom_map(&g, off + e * es + b)] = src[b];
        }
    }
    return 0;
}

/* ---- step 4 of the transfer: unpack ---------------------------------------- */

int hxo_unpack(const hxo_msg *m, const uint8_t *packed, int64_t B, int k,
               uint8_t *const *base, int nthreads)
{
    hxo_geom g;
    if (geom_init(&g, m, B, k)) return -1;
    (void)nthreads;
    for (int t = 0; t < m->T; ++t) {
        int64_t off = hxo_tensor_offset(m, t), n = hxo_tensor_elems(m, t);
        int es = m->esize[t];
#pragma omp parallel for num_threads(nthreads) schedule(static)
        for (int64_t e = 0; e < n; ++e) {
            uint8_t *dst = base[t] + hxo_element_storage_offset(m, t, e);
            for (int b = 0; b < es; ++b)
                dst[b] = packed[geom_map(&g, off + e * es + b)];
        }
    }
    return 0;
}

/* ---- widening: unpack that adds the arriving tensor to the one already there ----
 * The paper's Section 2.2 sends the intermediate results of a vendor-local reduction across
 * the boundary by the same P2P mechanism; the receiver combines them with its own.  Contract
 * chosen here (the paper gives none): per element, new = round(old + arriving), where
 *   kind 1 (bf16): both operands are widened exactly to binary32, added in binary32
 *                  (round to nearest even), and the binary32 sum is rounded to the nearest
 *                  bf16 value, ties to the value with an even last mantissa bit;
 *   kind 2 (f32) : IEEE binary32 addition, round to nearest even.
 * Any NaN result is stored as the canonical quiet NaN (bf16 0x7FC0, f32 0x7FC00000), so that
 * the outcome does not depend on how a machine propagates NaN payloads.
 * The bf16 rounding is written as the definition: scale the binary32 sum by a power of two so
 * that one bf16 unit in the last place becomes 1.0, round to an integer with ties to even,
 * scale back; double holds every intermediate exactly. */
#include <math.h>

static float bits_to_float(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static uint32_t float_to_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

uint16_t hxo_round_to_bf16(float x)
{
    if (isnan(x)) return 0x7FC0;
    if (isinf(x)) return x > 0 ? 0x7F80 : 0xFF80;
    double a = fabs((double)x);
    uint16_t sign = signbit(x) ? 0x8000 : 0;
    if (a == 0.0) return sign;
    int e;
    frexp(a, &e);                      /* a = m * 2^e, 0.5 <= m < 1: the leading bit has weight 2^(e-1) */
    int lead = e - 1;
    if (lead < -126) lead = -126;      /* subnormal range: fixed spacing */
    int ulp_exp = lead - 7;            /* bf16 keeps 7 fraction bits below the leading one */
    double q = nearbyint(ldexp(a, -ulp_exp));      /* default rounding mode: to nearest, ties to even */
    double r = ldexp(q, ulp_exp);                  /* the chosen bf16 value, exactly */
    if (r >= ldexp(1.0, 128)) return sign | 0x7F80;          /* rounded past the largest finite value */
    /* r is representable in binary32 with at most 8 significant bits: its top 16 bits are the answer */
    return sign | (uint16_t)(float_to_bits((float)r) >> 16);
}

uint32_t hxo_add_f32_bits(uint32_t a, uint32_t b)
{
    volatile float s = bits_to_float(a) + bits_to_float(b);
    if (isnan(s)) return 0x7FC00000u;
    return float_to_bits(s);
}

uint16_t hxo_add_bf16_bits(uint16_t a, uint16_t b)
{
    volatile float s = bits_to_float((uint32_t)a << 16) + bits_to_float((uint32_t)b << 16);
    return hxo_round_to_bf16(s);
}

/* kind[t]: 1 = bf16, 2 = f32 (element size must agree).  Returns -1 for anything else. */
int hxo_unpack_accumulate(const hxo_msg *m, const int32_t *kind, const uint8_t *packed, int64_t B, int k,
                          uint8_t *const *base, int nthreads)
{
    hxo_geom g;
    if (geom_init(&g, m, B, k)) return -1;
    for (int t = 0; t < m->T; ++t)
        if (!((kind[t] == 1 && m->esize[t] == 2) || (kind[t] == 2 && m->esize[t] == 4))) return -1;
    (void)nthreads;
    for (int t = 0; t < m->T; ++t) {
        int64_t off = hxo_tensor_offset(m, t), n = hxo_tensor_elems(m, t);
        int es = m->esize[t];
#pragma omp parallel for num_threads(nthreads) schedule(static)
        for (int64_t e = 0; e < n; ++e) {
            uint8_t *dst = base[t] + hxo_element_storage_offset(m, t, e);
            uint32_t in = 0, old = 0;
            for (int b = 0; b < es; ++b) {             /* little-endian element, byte by byte */
                in |= (uint32_t)packed[geom_map(&g, off + e * es + b)] << (8 * b);
                old |= (uint32_t)dst[b] << (8 * b);
            }
            uint32_t out = kind[t] == 1 ? hxo_add_bf16_bits((uint16_t)old, (uint16_t)in) : hxo_add_f32_bits(old, in);
            for (int b = 0; b < es; ++b) dst[b] = (uint8_t)(out >> (8 * b));
        }
    }
    return 0;
}

/* ---- step 3: staging one lane (device->host or host->device): identity ----- */

int hxo_stage_lane(int64_t L, int64_t B, int k, int l, const uint8_t *from, uint8_t *to)
{
    if (l < 0 || l >= k) return -1;
    int64_t off = hxo_lane_offset(L, B, k, l), used = hxo_lane_used(L, B, k, l);
    for (int64_t i = 0; i < used; ++i) to[off + i] = from[off + i];
    return 0;
}

/* Staging a run of slots of one lane: slots [first, first + count) of lane l, each up to the
 * padded end of the chunk it holds; slots past the lane's last chunk do not exist (-1). */
int hxo_stage_slots(int64_t L, int64_t B, int k, int l, int64_t first, int64_t count, const uint8_t *from, uint8_t *to)
{
    if (l < 0 || l >= k || first < 0 || count < 0) return -1;
    if (first + count > hxo_lane_chunks(L, B, k, l)) return -1;
    int64_t lane = hxo_lane_offset(L, B, k, l);
    for (int64_t s = first; s < first + count; ++s) {
        int64_t c = s * k + l;                        /* the chunk in slot s of lane l */
        int64_t off = lane + s * B, n = hxo_chunk_padded(L, B, c);
        for (int64_t i = 0; i < n; ++i) to[off + i] = from[off + i];
    }
    return 0;
}

/* ---- step 5: per-chunk checksum -------------------------------------------- */

int hxo_checksum(int64_t L, int64_t B, int k, const uint8_t *packed, uint64_t *sums, int nthreads)
{
    if (k < 1 || B <= 0 || B % HXO_ALIGN) return -1;
    int64_t C = hxo_num_chunks(L, B);
    (void)nthreads;
#pragma omp parallel for num_threads(nthreads) schedule(dynamic, 1)
    for (int64_t c = 0; c < C; ++c) {
        const uint8_t *p = packed + hxo_chunk_packed_offset(L, B, k, c);
        int64_t words = hxo_chunk_padded(L, B, c) / 4;
        uint64_t s = 0;
        for (int64_t j = 0; j < words; ++j) {
            uint32_t w = (uint32_t)p[4 * j] | (uint32_t)p[4 * j + 1] << 8 |
                         (uint32_t)p[4 * j + 2] << 16 | (uint32_t)p[4 * j + 3] << 24;
            s += w;
        }
        sums[c] = s;
    }
    return 0;
}

/* ---- widening: a second, position-weighted sum per chunk -----------------------
 * The plain sum cannot see words that changed places inside a chunk.  With the chunk's words
 * w_0 .. w_{W-1} (little-endian, W = padded length / 4), out[2c] = sum_j w_j and
 * out[2c+1] = sum_j (j+1) * w_j, both mod 2^64.  Swapping words i and j changes the second
 * sum by (j - i) * (w_i - w_j), which is non-zero mod 2^64 whenever the words differ. */
int hxo_checksum2(int64_t L, int64_t B, int k, const uint8_t *packed, uint64_t *out, int nthreads)
{
    if (k < 1 || B <= 0 || B % HXO_ALIGN) return -1;
    int64_t C = hxo_num_chunks(L, B);
    (void)nthreads;
#pragma omp parallel for num_threads(nthreads) schedule(dynamic, 1)
    for (int64_t c = 0; c < C; ++c) {
        const uint8_t *p = packed + hxo_chunk_packed_offset(L, B, k, c);
        int64_t words = hxo_chunk_padded(L, B, c) / 4;
        uint64_t s1 = 0, s2 = 0;
        for (int64_t j = 0; j < words; ++j) {
            uint64_t w = (uint64_t)p[4 * j] | (uint64_t)p[4 * j + 1] << 8 |
                         (uint64_t)p[4 * j + 2] << 16 | (uint64_t)p[4 * j + 3] << 24;
            s1 += w;
            s2 += (uint64_t)(j + 1) * w;
        }
        out[2 * c] = s1;
        out[2 * c + 1] = s2;
    }
    return 0;
}

/* ---- widening: chunk tags (a header per chunk that travels beside the lanes) ----------
 * The paper reports that mixed-vendor runs kept hanging until the transfer code was debugged
 * (subsection "Engineering Challenges"); a receiver that can tell WHICH message and which chunk
 * sits in a buffer turns a stale or misrouted ping-pong buffer into an error instead of a hang
 * or a silent mismatch.  The paper defines no header; this one is this repository's contract.
 *
 * One 64-byte record per chunk, all fields little-endian.  The record of chunk c is number
 * s(c) = packed offset of c / B in the tag array, i.e. the tags are in the order of the packed
 * slots, so that a lane's tags are one contiguous run like its chunks:
 *    byte  0  u32 magic = 0x31545848 (the bytes 'H','X','T','1')
 *    byte  4  u32 chunk index c
 *    byte  8  u32 lane(c)
 *    byte 12  u32 slot(c)
 *    byte 16  u64 seq          sender's running message number
 *    byte 24  u32 micro_batch  sender's micro-batch id
 *    byte 28  u32 C            chunks in the message
 *    byte 32  u64 padded(c)    bytes of the chunk that are transferred
 *    byte 40  u64 plain sum of the chunk's words      (as hxo_checksum2)
 *    byte 48  u64 position-weighted sum of its words  (as hxo_checksum2)
 *    byte 56  u64 zero
 * Verification of chunk c against the tag found at s(c) yields a bit mask, 0 = accepted: */
enum {
    HXO_TAG_BAD_MAGIC = 1,       /* magic differs */
    HXO_TAG_BAD_PLACE = 2,       /* chunk, lane, slot, C or padded differ from the receiver's own layout */
    HXO_TAG_BAD_SEQ = 4,         /* seq differs from the expected one */
    HXO_TAG_BAD_MICRO_BATCH = 8, /* micro_batch differs from the expected one */
    HXO_TAG_BAD_SUM = 16,        /* plain sum of the received bytes differs from the tag's */
    HXO_TAG_BAD_WSUM = 32,       /* weighted sum differs */
    HXO_TAG_BAD_RESERVED = 64    /* last field not zero */
};

static void hxo_put_le(uint8_t *p, int nbytes, uint64_t v)
{
    for (int i = 0; i < nbytes; ++i) p[i] = (uint8_t)(v >> (8 * i));
}

static uint64_t hxo_get_le(const uint8_t *p, int nbytes)
{
    uint64_t v = 0;
    for (int i = 0; i < nbytes; ++i) v |= (uint64_t)p[i] << (8 * i);
    return v;
}

/* tags: C * 64 bytes. */
int hxo_seal(int64_t L, int64_t B, int k, const uint8_t *packed, uint64_t seq, uint32_t micro_batch,
             uint8_t *tags)
{
    if (k < 1 || B <= 0 || B % HXO_ALIGN) return -1;
    int64_t C = hxo_num_chunks(L, B);
    for (int64_t c = 0; c < C; ++c) {
        const uint8_t *p = packed + hxo_chunk_packed_offset(L, B, k, c);
        int64_t words = hxo_chunk_padded(L, B, c) / 4;
        uint64_t s1 = 0, s2 = 0;
        for (int64_t j = 0; j < words; ++j) {
            uint64_t w = hxo_get_le(p + 4 * j, 4);
            s1 += w;
            s2 += (uint64_t)(j + 1) * w;
        }
        uint8_t *t = tags + 64 * (hxo_chunk_packed_offset(L, B, k, c) / B);
        hxo_put_le(t + 0, 4, 0x31545848u);
        hxo_put_le(t + 4, 4, (uint64_t)c);
        hxo_put_le(t + 8, 4, (uint64_t)hxo_chunk_lane(c, k));
        hxo_put_le(t + 12, 4, (uint64_t)hxo_chunk_slot(c, k));
        hxo_put_le(t + 16, 8, seq);
        hxo_put_le(t + 24, 4, micro_batch);
        hxo_put_le(t + 28, 4, (uint64_t)C);
        hxo_put_le(t + 32, 8, (uint64_t)hxo_chunk_padded(L, B, c));
        hxo_put_le(t + 40, 8, s1);
        hxo_put_le(t + 48, 8, s2);
        hxo_put_le(t + 56, 8, 0);
    }
    return 0;
}

/* status: C + 1 entries; status[c] = bit mask for chunk c, status[C] = number of chunks whose
 * mask is not zero. */
int hxo_verify(int64_t L, int64_t B, int k, const uint8_t *packed, const uint8_t *tags, uint64_t seq,
               uint32_t micro_batch, uint32_t *status)
{
    if (k < 1 || B <= 0 || B % HXO_ALIGN) return -1;
    int64_t C = hxo_num_chunks(L, B);
    uint32_t bad = 0;
    for (int64_t c = 0; c < C; ++c) {
        const uint8_t *p = packed + hxo_chunk_packed_offset(L, B, k, c);
        int64_t words = hxo_chunk_padded(L, B, c) / 4;
        uint64_t s1 = 0, s2 = 0;
        for (int64_t j = 0; j < words; ++j) {
            uint64_t w = hxo_get_le(p + 4 * j, 4);
            s1 += w;
            s2 += (uint64_t)(j + 1) * w;
        }
        const uint8_t *t = tags + 64 * (hxo_chunk_packed_offset(L, B, k, c) / B);
        uint32_t m = 0;
        if (hxo_get_le(t + 0, 4) != 0x31545848u) m |= HXO_TAG_BAD_MAGIC;
        if (hxo_get_le(t + 4, 4) != (uint64_t)c || hxo_get_le(t + 8, 4) != (uint64_t)hxo_chunk_lane(c, k) ||
            hxo_get_le(t + 12, 4) != (uint64_t)hxo_chunk_slot(c, k) || hxo_get_le(t + 28, 4) != (uint64_t)C ||
            hxo_get_le(t + 32, 8) != (uint64_t)hxo_chunk_padded(L, B, c))
            m |= HXO_TAG_BAD_PLACE;
        if (hxo_get_le(t + 16, 8) != seq) m |= HXO_TAG_BAD_SEQ;
        if (hxo_get_le(t + 24, 4) != micro_batch) m |= HXO_TAG_BAD_MICRO_BATCH;
        if (hxo_get_le(t + 40, 8) != s1) m |= HXO_TAG_BAD_SUM;
        if (hxo_get_le(t + 48, 8) != s2) m |= HXO_TAG_BAD_WSUM;
        if (hxo_get_le(t + 56, 8) != 0) m |= HXO_TAG_BAD_RESERVED;
        status[c] = m;
        if (m) ++bad;
    }
    status[C] = bad;
    return 0;
}

/* ---- inverse map, for sampled checks at sizes too big to pack on the CPU ---
 * Given a packed byte position p, say where it comes from:
 *   returns  1 and sets (*t, *storage_off): byte storage_off of tensor t's storage
 *   returns  0: a zero pad byte of the stream
 *   returns -1: unspecified (past the end of a short last chunk, or past packed_bytes)
 * Written from the layout description backwards (lane region -> slot -> chunk ->
 * stream byte -> tensor -> element), not by inverting hxo_pack's loop. */
int hxo_packed_origin(const hxo_msg *m, int64_t B, int k, int64_t p, int32_t *t_out, int64_t *storage_off)
{
    int64_t L = hxo_stream_bytes(m);
    if (p < 0 || p >= hxo_packed_bytes(L, B, k)) return -1;
    int l = 0;
    while (p >= hxo_lane_offset(L, B, k, l + 1)) ++l;
    int64_t within_lane = p - hxo_lane_offset(L, B, k, l);
    int64_t slot = within_lane / B, r = within_lane % B;
    int64_t c = slot * k + l;
    if (r >= hxo_chunk_padded(L, B, c)) return -1;
    int64_t s = c * B + r;
    for (int t = 0; t < m->T; ++t) {
        int64_t a = hxo_tensor_offset(m, t), n = hxo_tensor_bytes(m, t);
        if (s >= a && s < a + n) {
            int64_t e = (s - a) / m->esize[t], b = (s - a) % m->esize[t];
            *t_out = t;
            *storage_off = hxo_element_storage_offset(m, t, e) + b;
            return 1;
        }
    }
    return 0;
}

int hxo_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
