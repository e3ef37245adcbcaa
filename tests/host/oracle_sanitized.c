/* Test helper: the CPU oracle compiled into one program with AddressSanitizer and
 * UndefinedBehaviorSanitizer and driven over small messages whose buffers are allocated at
 * exactly the size each call may touch, so that any access outside them aborts the run.
 * It checks the round trip and the agreement of the oracle's own entry points with each
 * other; what the oracle's values should BE is pinned elsewhere (tests/test_oracle_*.py). */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../oracle/hxt_oracle.c"

#define EXPECT(cond)                                                          \
    do {                                                                      \
        if (!(cond)) {                                                        \
            printf("oracle_sanitized: line %d: %s\n", __LINE__, #cond);       \
            exit(1);                                                          \
        }                                                                     \
    } while (0)

typedef struct {
    int ndim;
    int64_t shape[HXO_MAXDIM], stride[HXO_MAXDIM];
    int esize;
} view;

static int64_t storage_bytes(const view *v)
{
    int64_t reach = 0;
    for (int d = 0; d < v->ndim; ++d) {
        if (v->shape[d] == 0) return 0;
        reach += (v->shape[d] - 1) * v->stride[d];
    }
    return (reach + 1) * v->esize;
}

static uint8_t *exact(int64_t n)          /* n bytes, never NULL, nothing to spare */
{
    uint8_t *p = malloc(n > 0 ? (size_t)n : 1);
    EXPECT(p != NULL);
    return p;
}

static void run(const view *vs, int T, int64_t B, int k, int aliasing)
{
    int32_t ndim[8], esize[8];
    int64_t shape[8 * HXO_MAXDIM] = {0}, stride[8 * HXO_MAXDIM] = {0};
    uint8_t *src[8], *dst[8];
    for (int t = 0; t < T; ++t) {
        ndim[t] = vs[t].ndim;
        esize[t] = vs[t].esize;
        for (int d = 0; d < vs[t].ndim; ++d) {
            shape[t * HXO_MAXDIM + d] = vs[t].shape[d];
            stride[t * HXO_MAXDIM + d] = vs[t].stride[d];
        }
        int64_t n = storage_bytes(&vs[t]);
        src[t] = exact(n);
        dst[t] = exact(n);
        for (int64_t i = 0; i < n; ++i) src[t][i] = (uint8_t)(rand() >> 7);
        memset(dst[t], 0x3C, n > 0 ? (size_t)n : 1);
    }
    hxo_msg m = {T, ndim, shape, stride, esize};
    int64_t L = hxo_stream_bytes(&m), C = hxo_num_chunks(L, B), P = hxo_packed_bytes(L, B, k);
    EXPECT(P == C * B);
    uint8_t *packed = exact(P), *host = exact(P), *recv = exact(P);
    memset(packed, 0xA5, P > 0 ? (size_t)P : 1);
    memset(host, 0, P > 0 ? (size_t)P : 1);
    memset(recv, 0x5A, P > 0 ? (size_t)P : 1);
    EXPECT(hxo_pack(&m, (const uint8_t *const *)src, B, k, packed, 1) == 0);
    int64_t payload = 0;
    for (int64_t c = 0; c < C; ++c) payload += hxo_chunk_payload(&m, B, c);
    EXPECT(payload == hxo_message_bytes(&m));
    uint64_t *sums = (uint64_t *)exact(8 * C), *sums2 = (uint64_t *)exact(16 * C);
    EXPECT(hxo_checksum(L, B, k, packed, sums, 1) == 0);
    EXPECT(hxo_checksum2(L, B, k, packed, sums2, 1) == 0);
    for (int64_t c = 0; c < C; ++c) EXPECT(sums2[2 * c] == sums[c]);
    uint8_t *tags = exact(64 * C);
    uint32_t *status = (uint32_t *)exact(4 * (C + 1));
    EXPECT(hxo_seal(L, B, k, packed, 77, 5, tags) == 0);
    EXPECT(hxo_verify(L, B, k, packed, tags, 77, 5, status) == 0);
    for (int64_t c = 0; c <= C; ++c) EXPECT(status[c] == 0);
    for (int l = 0; l < k; ++l) {                       /* the CPU-forwarding leg, lane by lane */
        EXPECT(hxo_stage_lane(L, B, k, l, packed, host) == 0);
        EXPECT(hxo_stage_lane(L, B, k, l, host, recv) == 0);
    }
    EXPECT(hxo_verify(L, B, k, recv, tags, 77, 5, status) == 0);
    EXPECT(status[C] == 0);
    memset(recv, 0x5A, (size_t)(P > 0 ? P : 1));         /* and slot by slot */
    for (int l = 0; l < k; ++l) {
        int64_t n = hxo_lane_chunks(L, B, k, l);
        for (int64_t s = 0; s < n; ++s) EXPECT(hxo_stage_slots(L, B, k, l, s, 1, host, recv) == 0);
        EXPECT(hxo_stage_slots(L, B, k, l, n, 1, host, recv) == -1);
    }
    EXPECT(hxo_verify(L, B, k, recv, tags, 77, 5, status) == 0);
    EXPECT(status[C] == 0);
    for (int64_t p = 0; p < P; ++p) {                   /* every packed byte has an origin, and it is the right one */
        int32_t t = -1;
        int64_t off = -1;
        int kind = hxo_packed_origin(&m, B, k, p, &t, &off);
        if (kind == 1) EXPECT(t >= 0 && t < T && off >= 0 && off < storage_bytes(&vs[t]) && packed[p] == src[t][off]);
        if (kind == 0) EXPECT(packed[p] == 0);
        if (kind == -1) EXPECT(packed[p] == 0xA5 && recv[p] == 0x5A);
    }
    if (!aliasing) {
        EXPECT(hxo_unpack(&m, recv, B, k, dst, 1) == 0);
        uint8_t *again = exact(P);
        memset(again, 0xA5, P > 0 ? (size_t)P : 1);
        EXPECT(hxo_pack(&m, (const uint8_t *const *)dst, B, k, again, 1) == 0);
        EXPECT(memcmp(again, packed, (size_t)P) == 0);  /* what arrived packs to the same bytes */
        free(again);
    }
    for (int t = 0; t < T; ++t) {
        free(src[t]);
        free(dst[t]);
    }
    free(packed); free(host); free(recv); free(sums); free(sums2); free(tags); free(status);
}

int main(void)
{
    srand(18007);
    const view contig_u8 = {1, {1000}, {1}, 1};
    const view bf16_2d = {2, {17, 33}, {33, 1}, 2};
    const view rows = {2, {7, 100}, {128, 1}, 2};
    const view interleaved = {3, {6, 2, 64}, {64, 384, 1}, 2};
    const view transposed = {2, {64, 48}, {1, 64}, 2};
    const view f32_t = {2, {33, 17}, {1, 40}, 4};
    const view broadcast = {2, {5, 64}, {0, 1}, 4};
    const view f64 = {2, {12, 10}, {16, 1}, 8};
    const view scalar = {0, {0}, {0}, 4};
    const view empty = {2, {0, 16}, {16, 1}, 2};
    const view eight = {8, {2, 3, 2, 2, 3, 2, 2, 4}, {288, 48, 2, 576, 4, 1, 144, 12}, 2};
    const int64_t Bs[] = {256, 512, 4096};
    const int ks[] = {1, 2, 3, 8};
    const view singles[] = {contig_u8, bf16_2d, rows, interleaved, transposed, f32_t, f64, scalar, empty, eight};
    for (size_t b = 0; b < sizeof Bs / sizeof *Bs; ++b)
        for (size_t j = 0; j < sizeof ks / sizeof *ks; ++j) {
            for (size_t i = 0; i < sizeof singles / sizeof *singles; ++i) run(&singles[i], 1, Bs[b], ks[j], 0);
            run(&broadcast, 1, Bs[b], ks[j], 1);
            const view multi[] = {contig_u8, empty, rows, transposed, f64, scalar};
            run(multi, 6, Bs[b], ks[j], 0);
        }
    /* receive and accumulate on exactly sized bf16 and f32 buffers */
    {
        int32_t ndim[2] = {1, 1}, esize[2] = {2, 4}, kind[2] = {1, 2};
        int64_t shape[2 * HXO_MAXDIM] = {0}, stride[2 * HXO_MAXDIM] = {0};
        shape[0] = 301; stride[0] = 1; shape[HXO_MAXDIM] = 77; stride[HXO_MAXDIM] = 1;
        hxo_msg m = {2, ndim, shape, stride, esize};
        int64_t L = hxo_stream_bytes(&m), P = hxo_packed_bytes(L, 512, 3);
        uint8_t *a = exact(602), *b = exact(308), *packed = exact(P);
        for (int i = 0; i < 602; ++i) a[i] = (uint8_t)(rand() >> 7);
        for (int i = 0; i < 308; ++i) b[i] = (uint8_t)(rand() >> 7);
        const uint8_t *src[2] = {a, b};
        uint8_t *dst[2] = {a, b};
        EXPECT(hxo_pack(&m, src, 512, 3, packed, 1) == 0);
        EXPECT(hxo_unpack_accumulate(&m, kind, packed, 512, 3, dst, 1) == 0);
        free(a); free(b); free(packed);
    }
    printf("oracle_sanitized: ok\n");
    return 0;
}
