/* A plain C99 caller of the boundary (include/spmm.h) that runs the product on the
 * device: spmm_plan_create -> spmm_execute -> spmm_plan_destroy, with device memory
 * from the HIP runtime's C interface (declared by hand: no HIP header, no C++).
 * Built and run by tests/test_gpu_parity.py on the GPU machine.
 *
 * A = [ 1 0 0 2 ]     B[k][j] = 10 k + j (4 x 8)
 *     [ 0 0 0 0 ]
 *     [ 0 3 0 0 ]     C[0][j] = 1 (0 + j) + 2 (30 + j) = 60 + 3 j
 *                     C[1][j] = 0,  C[2][j] = 3 (10 + j) = 30 + 3 j
 */
#include <stddef.h>
#include <stdio.h>
#include "spmm.h"

extern int hipMalloc(void **ptr, size_t bytes);
extern int hipFree(void *ptr);
extern int hipMemcpy(void *dst, const void *src, size_t bytes, int kind); /* 1 = host to device, 2 = device to host */
extern int hipDeviceSynchronize(void);

int main(void) {
    int32_t row_ptr[4] = {0, 2, 2, 3};
    int32_t col_idx[3] = {0, 3, 1};
    float vals[3] = {1.f, 2.f, 3.f};
    float B[4 * 8], C[3 * 8];
    void *dB = NULL, *dC = NULL;
    spmm_plan_t *p = NULL;
    spmm_status_t st;
    int k, j, bad = 0;
    for (k = 0; k < 4; ++k)
        for (j = 0; j < 8; ++j) B[k * 8 + j] = (float)(10 * k + j);
    for (j = 0; j < 3 * 8; ++j) C[j] = -1.f;
    if (hipMalloc(&dB, sizeof B) != 0 || hipMalloc(&dC, sizeof C) != 0) { printf("hipMalloc failed\n"); return 1; }
    if (hipMemcpy(dB, B, sizeof B, 1) != 0 || hipMemcpy(dC, C, sizeof C, 1) != 0) { printf("upload failed\n"); return 1; }
    st = spmm_plan_create(&p, 3, 4, row_ptr, col_idx, vals);
    if (st != SPMM_OK) { printf("create: %s\n", spmm_status_string(st)); return 2; }
    st = spmm_execute(p, (const float *)dB, 8, (float *)dC, NULL);
    if (st != SPMM_OK) { printf("execute: %s\n", spmm_status_string(st)); return 3; }
    if (hipDeviceSynchronize() != 0 || hipMemcpy(C, dC, sizeof C, 2) != 0) { printf("download failed\n"); return 4; }
    for (j = 0; j < 8; ++j) {
        if (C[j] != (float)(60 + 3 * j)) bad++;
        if (C[8 + j] != 0.f) bad++;
        if (C[16 + j] != (float)(30 + 3 * j)) bad++;
    }
    printf("C[0][0]=%g C[0][7]=%g C[2][5]=%g mismatches=%d\n", (double)C[0], (double)C[7], (double)C[16 + 5], bad);
    st = spmm_plan_destroy(p);
    (void)hipFree(dB);
    (void)hipFree(dC);
    if (bad == 0 && st == SPMM_OK) printf("device client ok\n");
    return bad == 0 && st == SPMM_OK ? 0 : 5;
}
