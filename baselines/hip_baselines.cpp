// Comparison systems for bench.py (not part of the product path): hipSPARSE CSR
// SpMM and rocBLAS SGEMM on device-resident inputs, timed with HIP events.
// Both are given their best shot: row-major B and C, every CSR SpMM algorithm
// the header offers, buffer-size and preprocess calls outside the timed region.
#include <hip/hip_runtime_api.h>
#include <hipsparse/hipsparse.h>
#include <rocblas/rocblas.h>

#include <algorithm>
#include <chrono>
#include <cstdio>
#include <vector>

namespace {

// median over `samples` of (time of `inner` back-to-back calls) / inner, in ms;
// *mean_out (may be null) receives the mean over the samples
template <typename F> float time_ms(F &&call, int samples, int inner, float *mean_out = nullptr)
{
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return -1.f;
    // warm up for at least 10 ms of queued work: after an idle spell the clocks need that long
    const auto t0 = std::chrono::steady_clock::now();
    do {
        for (int i = 0; i < inner; ++i) call();
        (void)hipDeviceSynchronize();
    } while (std::chrono::steady_clock::now() - t0 < std::chrono::milliseconds(10));
    std::vector<float> t;
    for (int s = 0; s < samples; ++s) {
        (void)hipEventRecord(a, nullptr);
        for (int i = 0; i < inner; ++i) call();
        (void)hipEventRecord(b, nullptr);
        (void)hipEventSynchronize(b);
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, a, b);
        t.push_back(ms / inner);
    }
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    std::sort(t.begin(), t.end());
    if (mean_out) {
        double sum = 0;
        for (float x : t) sum += x;
        *mean_out = (float)(sum / (double)t.size());
    }
    return t[t.size() / 2];
}

}  // namespace

extern "C" {

// All pointers DEVICE except ms_out (HOST, 4 floats: one per algorithm, -1 = not run).
// Returns 0 on success.
int baseline_hipsparse_spmm(int M, int K, int N, int nnz, const int *row_ptr, const int *col_idx,
                            const float *vals, const float *B, float *C, int samples, int inner,
                            float *ms_out)
{
    hipsparseHandle_t h;
    if (hipsparseCreate(&h) != HIPSPARSE_STATUS_SUCCESS) return 1;
    hipsparseSpMatDescr_t A;
    hipsparseDnMatDescr_t Bd, Cd;
    int rc = 0;
    if (hipsparseCreateCsr(&A, M, K, nnz, (void *)row_ptr, (void *)col_idx, (void *)vals, HIPSPARSE_INDEX_32I,
                           HIPSPARSE_INDEX_32I, HIPSPARSE_INDEX_BASE_ZERO, HIP_R_32F) != HIPSPARSE_STATUS_SUCCESS)
        rc = 2;
    if (!rc && hipsparseCreateDnMat(&Bd, K, N, N, (void *)B, HIP_R_32F, HIPSPARSE_ORDER_ROW) != HIPSPARSE_STATUS_SUCCESS)
        rc = 3;
    if (!rc && hipsparseCreateDnMat(&Cd, M, N, N, (void *)C, HIP_R_32F, HIPSPARSE_ORDER_ROW) != HIPSPARSE_STATUS_SUCCESS)
        rc = 4;
    const hipsparseSpMMAlg_t algs[4] = {HIPSPARSE_SPMM_ALG_DEFAULT, HIPSPARSE_SPMM_CSR_ALG1, HIPSPARSE_SPMM_CSR_ALG2,
                                        HIPSPARSE_SPMM_CSR_ALG3};
    const float alpha = 1.f, beta = 0.f;
    for (int i = 0; i < 4 && !rc; ++i) {
        ms_out[i] = -1.f;
        size_t bytes = 0;
        if (hipsparseSpMM_bufferSize(h, HIPSPARSE_OPERATION_NON_TRANSPOSE, HIPSPARSE_OPERATION_NON_TRANSPOSE, &alpha, A,
                                     Bd, &beta, Cd, HIP_R_32F, algs[i], &bytes) != HIPSPARSE_STATUS_SUCCESS)
            continue;
        void *buf = nullptr;
        if (bytes && hipMalloc(&buf, bytes) != hipSuccess) continue;
        if (hipsparseSpMM_preprocess(h, HIPSPARSE_OPERATION_NON_TRANSPOSE, HIPSPARSE_OPERATION_NON_TRANSPOSE, &alpha, A,
                                     Bd, &beta, Cd, HIP_R_32F, algs[i], buf) == HIPSPARSE_STATUS_SUCCESS) {
            bool ok = true;
            auto call = [&]() {
                if (hipsparseSpMM(h, HIPSPARSE_OPERATION_NON_TRANSPOSE, HIPSPARSE_OPERATION_NON_TRANSPOSE, &alpha, A, Bd,
                                  &beta, Cd, HIP_R_32F, algs[i], buf) != HIPSPARSE_STATUS_SUCCESS)
                    ok = false;
            };
            const float ms = time_ms(call, samples, inner);
            if (ok) ms_out[i] = ms;
        }
        if (buf) (void)hipFree(buf);
    }
    if (rc == 0 || rc > 4) (void)hipsparseDestroyDnMat(Cd);
    if (rc == 0 || rc > 3) (void)hipsparseDestroyDnMat(Bd);
    if (rc == 0 || rc > 2) (void)hipsparseDestroySpMat(A);
    (void)hipsparseDestroy(h);
    return rc;
}

// C (M x N, row-major) = A (M x K, row-major, dense) x B (K x N, row-major), fp32.
// Row-major product through the column-major routine: C^T = B^T A^T.
int baseline_rocblas_sgemm(int M, int K, int N, const float *A, const float *B, float *C, int samples, int inner,
                           float *ms_out)
{
    rocblas_handle h;
    if (rocblas_create_handle(&h) != rocblas_status_success) return 1;
    const float alpha = 1.f, beta = 0.f;
    bool ok = true;
    auto call = [&]() {
        if (rocblas_sgemm(h, rocblas_operation_none, rocblas_operation_none, N, M, K, &alpha, B, N, A, K, &beta, C, N) !=
            rocblas_status_success)
            ok = false;
    };
    *ms_out = time_ms(call, samples, inner);
    (void)rocblas_destroy_handle(h);
    return ok ? 0 : 2;
}

// The library under test timed the same way as the two comparison systems: `fn` is
// its spmm_execute (signature of include/spmm.h, status 0 = ok), called on the default
// stream from this C loop so that no interpreter sits between two launches.
// ms_out: HOST, 2 floats (median, mean).
typedef int (*spmm_execute_fn)(const void *plan, const float *B, int N, float *C, void *stream);
int baseline_time_spmm_execute(spmm_execute_fn fn, const void *plan, const float *B, int N, float *C,
                               int samples, int inner, float *ms_out)
{
    bool ok = true;
    auto call = [&]() {
        if (fn(plan, B, N, C, nullptr) != 0) ok = false;
    };
    ms_out[0] = time_ms(call, samples, inner, &ms_out[1]);
    return ok ? 0 : 2;
}

// The same loop over `copies` independent (plan, B, C) triples taken in turn, so that a
// call finds none of its operands in the caches when the triples together exceed them.
int baseline_time_spmm_execute_rotating(spmm_execute_fn fn, const void *const *plans, const float *const *Bs,
                                        float *const *Cs, int copies, int N, int samples, int inner, float *ms_out)
{
    if (copies < 1) return 1;
    bool ok = true;
    int next = 0;
    auto call = [&]() {
        if (fn(plans[next], Bs[next], N, Cs[next], nullptr) != 0) ok = false;
        next = next + 1 == copies ? 0 : next + 1;
    };
    ms_out[0] = time_ms(call, samples, inner, &ms_out[1]);
    return ok ? 0 : 2;
}

}  // extern "C"
