/*
 * The boundary used from plain C (no Python, no C++): builds a plan through include/rose_delta.h,
 * asks the host-side queries and checks a few answers.  Needs no GPU: no device call is made.
 * Built with gcc -std=c99 -pedantic and linked against librose_delta.so by tests/test_c_abi.py.
 */
#include <stdio.h>
#include <string.h>

#include "rose_delta.h"

int main(void)
{
    rose_tensor_desc t[3];
    rose_plan *plan = NULL;
    int64_t v = 0;
    size_t bytes = 0;
    int32_t d = -1, n = -1, local = -1;

    memset(t, 0, sizeof t);
    t[0].rows = 1;  t[0].cols = 4096; t[0].rule = ROSE_REPLICATED;
    t[1].rows = 64; t[1].cols = 512;  t[1].rule = ROSE_SPLIT_COLS;
    t[2].rows = 96; t[2].cols = 256;  t[2].rule = ROSE_FUSED_ROWS;
    t[2].n_sections = 3; t[2].section_rows[0] = 64; t[2].section_rows[1] = 16; t[2].section_rows[2] = 16;

    if (rose_shard_plan_create(t, 3, 4, &plan) != ROSE_OK || !plan) { printf("create failed\n"); return 1; }
    if (rose_plan_n_tensors(plan) != 3 || rose_plan_tp(plan) != 4) { printf("counts\n"); return 1; }
    if (rose_plan_local_numel(plan, 1, 2, &v) != ROSE_OK || v != 64 * 128) { printf("local numel\n"); return 1; }
    if (rose_plan_tensor_base(plan, 2, &v) != ROSE_OK || v != 4096 + 64 * 512) { printf("base\n"); return 1; }
    if (rose_plan_bucket_capacity(plan, 0, &v) != ROSE_OK || v != 4096 + 64 * 128 + 24 * 256) { printf("capacity\n"); return 1; }
    if (rose_plan_workspace_bytes(plan, &bytes) != ROSE_OK || bytes == 0) { printf("workspace\n"); return 1; }
    /* element (row 3, column 300) of the column-split matrix: shard 2, local row 3, local column 44 */
    if (rose_plan_map_index(plan, 1, 3 * 512 + 300, &d, &n, &local) != ROSE_OK || d != 2 || n != 1 || local != 3 * 128 + 44) {
        printf("map %d %d %d\n", d, n, local);
        return 1;
    }
    /* row 70 of the fused matrix is row 6 of the second section: shard 1, local row 16 + 2 */
    if (rose_plan_map_index(plan, 2, 70 * 256 + 5, &d, &n, &local) != ROSE_OK || d != 1 || n != 1 || local != 18 * 256 + 5) {
        printf("fused map %d %d %d\n", d, n, local);
        return 1;
    }
    if (rose_plan_map_index(plan, 0, 17, &d, &n, &local) != ROSE_OK || d != 0 || n != 4 || local != 17) { printf("replicated\n"); return 1; }
    if (strcmp(rose_status_str(ROSE_ERR_CAPACITY), rose_status_str(ROSE_OK)) == 0) { printf("status strings\n"); return 1; }
    rose_shard_plan_destroy(plan);
    printf("ok\n");
    return 0;
}
