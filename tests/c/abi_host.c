/* Plain C99 caller of the C ABI (no GPU needed): a host-only plan from two explicit segments,
 * its manifest queries, and the synchronous error paths.  Exits 0 when every check holds. */
#include <stdio.h>
#include <string.h>
#include "th.h"

#define CHECK(c) do { if (!(c)) { fprintf(stderr, "line %d: %s (last error: %s)\n", __LINE__, #c, th_last_error()); return 1; } } while (0)

int main(void) {
    th_segment seg[2];
    memset(seg, 0, sizeof seg);
    /* tensor 0: 3 rows of 10 fp32 elements out of rows of 12, narrowed to bf16, dense destination */
    seg[0].src_tensor = 0; seg[0].dst_tensor = 0;
    seg[0].src_elem_off = 1; seg[0].src_row_stride = 12; seg[0].dst_elem_off = 0; seg[0].dst_row_stride = 10;
    seg[0].nrows = 3; seg[0].row_len = 10; seg[0].src_dtype = TH_F32; seg[0].dst_dtype = TH_BF16;
    /* tensor 1: one row of 7 bf16 elements */
    seg[1].src_tensor = 1; seg[1].dst_tensor = 0;
    seg[1].src_elem_off = 0; seg[1].src_row_stride = 7; seg[1].dst_elem_off = 30; seg[1].dst_row_stride = 7;
    seg[1].nrows = 1; seg[1].row_len = 7; seg[1].src_dtype = TH_BF16; seg[1].dst_dtype = TH_BF16;
    const uint64_t src_elems[2] = {40, 7}, dst_elems[1] = {37};
    th_plan* plan = NULL;
    CHECK(th_plan_create_from_segments(seg, 2, src_elems, 2, dst_elems, 1, 32, TH_FLAG_HOST_ONLY, &plan) == TH_OK);
    CHECK(plan != NULL);
    /* wire: 30 bf16 = 60 bytes, gap to 64, then 7 bf16 = 14 bytes */
    CHECK(th_plan_payload_bytes(plan) == 74);
    CHECK(th_plan_wire_bytes(plan) == 78);
    CHECK(th_plan_num_chunks(plan) == 3);
    CHECK(th_plan_chunk_bytes(plan, 0) == 32 && th_plan_chunk_bytes(plan, 2) == 14);
    CHECK(th_plan_num_tensors(plan, 0) == 2 && th_plan_num_tensors(plan, 1) == 1);
    CHECK(th_plan_num_runs(plan) >= 3);
    /* a host-only plan refuses to launch, synchronously */
    const void* srcs[2] = {NULL, NULL};
    void* wire[1] = {NULL};
    CHECK(th_pack(plan, srcs, 2, wire, 0, 1, NULL) == TH_ERR_ARG);
    CHECK(strlen(th_last_error()) > 0);
    CHECK(th_plan_destroy(plan) == TH_OK);
    CHECK(th_plan_destroy(NULL) == TH_OK);
    /* argument errors */
    plan = NULL;
    CHECK(th_plan_create_from_segments(seg, 2, src_elems, 2, dst_elems, 1, 30, TH_FLAG_HOST_ONLY, &plan) == TH_ERR_ARG);
    seg[0].nrows = 4; /* reaches outside the source tensor */
    CHECK(th_plan_create_from_segments(seg, 2, src_elems, 2, dst_elems, 1, 32, TH_FLAG_HOST_ONLY, &plan) == TH_ERR_RANGE);
    CHECK(th_version() != NULL);
    printf("c abi ok\n");
    return 0;
}
