/* A plain C client of the library (test helper): control-plane calls only, so that it runs
 * with or without a GPU.  Exits 0 if every answer is the expected one, else prints the
 * failing line and exits 1.  Expected values are those of the LLaMA-shaped boundary message
 * written out by hand: 4096 * 1 * 4096 bf16 = 33 554 432 bytes, 1 MiB chunks -> 32 chunks,
 * 4 lanes -> 8 chunks per lane, lane l starting at l * 8 MiB. */
#include <stdio.h>
#include <string.h>

#include "hxt.h"

#define EXPECT(cond)                                                    \
    do {                                                                \
        if (!(cond)) {                                                  \
            printf("abi_client: line %d: %s\n", __LINE__, #cond);       \
            return 1;                                                   \
        }                                                               \
    } while (0)

int main(void)
{
    const int64_t shape[3] = {4096, 1, 4096};
    const int64_t strides[3] = {4096, 16777216, 1};          /* [seq, mb, hidden] view of [mb, seq, hidden] */
    hxt_plan_t *plan = NULL;
    EXPECT(hxt_plan(shape, strides, 3, HXT_BF16, 4, 1u << 20, &plan) == HXT_OK);
    EXPECT(plan != NULL);
    EXPECT(hxt_plan_message_bytes(plan) == 33554432u);
    EXPECT(hxt_plan_stream_bytes(plan) == 33554432u);
    EXPECT(hxt_plan_packed_bytes(plan) == 33554432u);
    EXPECT(hxt_plan_chunk_bytes(plan) == (1u << 20));
    EXPECT(hxt_plan_num_chunks(plan) == 32);
    EXPECT(hxt_plan_num_lanes(plan) == 4);
    EXPECT(hxt_plan_num_tensors(plan) == 1);
    EXPECT(hxt_plan_tensor_unpack_safe(plan, 0) == 1);
    for (int l = 0; l < 4; ++l) {
        hxt_lane_info_t li;
        EXPECT(hxt_plan_lane_info(plan, l, &li) == HXT_OK);
        EXPECT(li.n_chunks == 8 && li.bytes == (8u << 20) && li.packed_off == (uint64_t)l * (8u << 20));
    }
    hxt_chunk_info_t ci;
    EXPECT(hxt_plan_chunk_info(plan, 6, &ci) == HXT_OK);     /* chunk 6: lane 2, slot 1 */
    EXPECT(ci.lane == 2 && ci.slot == 1 && ci.stream_off == (6u << 20) && ci.padded == (1u << 20));
    EXPECT(ci.payload == (1u << 20) && ci.packed_off == (2u * 8u + 1u) * (1u << 20));
    EXPECT(hxt_plan_chunk_info(plan, 32, &ci) == HXT_EINVAL);
    EXPECT(hxt_plan_lane_info(plan, 4, NULL) == HXT_EINVAL);
    EXPECT(hxt_plan_set_option(plan, HXT_OPT_PACKED_HINT, 1) == HXT_OK);
    EXPECT(hxt_plan_set_option(plan, HXT_OPT_STAGE_D2H, 7) == HXT_EINVAL);
    EXPECT(hxt_stage_d2h_slots(plan, 1, 7, 2, NULL, NULL, NULL) == HXT_EINVAL);   /* lane 1 has slots 0..7 */
    EXPECT(hxt_stage_h2d_slots(plan, 1, 8, 0, NULL, NULL, NULL) == HXT_OK);       /* the empty run */
    hxt_exchange_t x;
    memset(&x, 0, sizeof x);
    x.n_messages = 1;
    x.n_buffers = 2;
    x.direct_mode = 9;
    EXPECT(hxt_exchange_stream(plan, &x) == HXT_EINVAL);
    EXPECT(hxt_pack_noalloc(NULL, 0, 4, 1u << 20, NULL, NULL, NULL) == HXT_OK);
    EXPECT(hxt_pack_noalloc(NULL, 64, 4, 1000, NULL, NULL, NULL) == HXT_EINVAL);
    EXPECT(hxt_plan_destroy(plan) == HXT_OK);
    EXPECT(hxt_plan_destroy(NULL) == HXT_OK);

    plan = NULL;
    EXPECT(hxt_plan(shape, strides, 3, HXT_BF16, 0, 1u << 20, &plan) == HXT_EINVAL && plan == NULL);
    EXPECT(hxt_plan(shape, strides, 3, HXT_BF16, 4, 1000, &plan) == HXT_EINVAL && plan == NULL);
    EXPECT(hxt_plan(shape, strides, 3, HXT_BF16, 4, 1u << 20, NULL) == HXT_EINVAL);
    EXPECT(hxt_pack(NULL, NULL, NULL, NULL, NULL) == HXT_EINVAL);
    EXPECT(strcmp(hxt_strerror(HXT_OK), "ok") == 0);
    EXPECT(strlen(hxt_strerror(HXT_EOVERLAP)) > 0 && strlen(hxt_version()) > 0);
    EXPECT(sizeof(hxt_chunk_tag_t) == 64);
    printf("abi_client: ok (%s)\n", hxt_version());
    return 0;
}
