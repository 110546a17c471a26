/* A plain C99 client of the boundary (include/spmm.h): compiled and run by
 * tests/test_c_abi_client.py.  Builds a plan in host memory (no device needed),
 * reads it back and checks that a host-only plan refuses to execute. */
#include <stdio.h>
#include "spmm.h"
int main(void) {
    int32_t row_ptr[4] = {0, 2, 2, 3};
    int32_t col_idx[3] = {0, 3, 1};
    float vals[3] = {1.f, 2.f, 3.f};
    spmm_options_t o = {0};
    o.host_only = 1;
    spmm_plan_t *p = NULL;
    spmm_status_t st = spmm_plan_create_ex(&p, 3, 4, row_ptr, col_idx, vals, &o);
    if (st != SPMM_OK) { printf("create: %s\n", spmm_status_string(st)); return 1; }
    spmm_plan_info_t info;
    st = spmm_plan_describe(p, &info);
    printf("M=%lld K=%lld nnz=%lld ufi=%d groups=%lld blocks=%lld\n", (long long)info.M, (long long)info.K, (long long)info.nnz, info.ufi, (long long)info.n_groups, (long long)info.n_blocks);
    st = spmm_execute(p, NULL, 4, NULL, NULL);
    printf("execute on host-only plan: %s\n", spmm_status_string(st));
    return spmm_plan_destroy(p) == SPMM_OK ? 0 : 2;
}
