/* The headers are plain C: this file is compiled with gcc -std=c99 -pedantic -Werror,
 * linked against libkvl.so and run without a GPU (host-only plan, scheduling functions). */
#include <stdio.h>
#include <string.h>

#include "kvl.h"
#include "kvl_sched.h"

int main(void) {
    kvl_layout_t lay;
    int32_t t0[3] = {1, 2, 3}, t1[1] = {5};
    kvl_request_t req[2];
    kvl_plan_t *plan = NULL;
    kvl_unit_t units[8];
    uint64_t n = 0, bytes = 0;
    kvl_pd_range_t range;
    memset(&lay, 0, sizeof lay);
    lay.n_layers = 2; lay.block_tokens = 4; lay.n_planes = 2; lay.row_bytes[0] = 16; lay.row_bytes[1] = 32;
    lay.pool_blocks = 10;
    req[0].hit_tokens = 9; req[0].append_tokens = 1; req[0].n_blocks = 3; req[0].block_table = t0;
    req[1].hit_tokens = 2; req[1].append_tokens = 2; req[1].n_blocks = 1; req[1].block_table = t1;
    if (kvl_plan(&lay, req, 2, KVL_GATHER | KVL_HOST_ONLY, &plan) != KVL_OK) return 1;
    if (kvl_plan_payload_bytes(plan, &bytes) != KVL_OK || bytes != 11u * 48u) return 2;
    if (kvl_plan_get_units(plan, units, 8, &n) != KVL_OK || n != 2) return 3;
    if (units[0].pool_row != 4 || units[0].n_rows != 9 || units[1].pool_row != 20 || units[1].xfer_row != 9) return 4;
    if (kvl_pack_layer(plan, NULL, NULL, 0, NULL) != KVL_EINVAL) return 5;   /* a host-only plan cannot run */
    kvl_plan_destroy(plan);
    if (kvl_pd_range(8, 1, 500, 50, &range) != KVL_OK || !range.feasible) return 6;
    if (kvl_sched_read_side(3, 2) != 1 || kvl_sched_read_side(2, 2) != 0) return 7;
    if (strcmp(kvl_strerror(KVL_EALIAS), kvl_strerror(KVL_ESPACE)) == 0) return 8;
    printf("c abi ok: %s\n", kvl_version());
    return 0;
}
