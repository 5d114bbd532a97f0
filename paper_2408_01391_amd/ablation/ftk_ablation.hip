// Measurement-only kernels: the steps of Section 3.1 that precede the fused kernel.
#include <hip/hip_runtime.h>
#include <rocblas/rocblas.h>

#include <cstdarg>
#include <cstdio>

#include "ftk_ablation.h"

namespace {

thread_local char g_err[256] = "";

void set_err(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
}

// Section 3.1.1: a thread owns a point; for each centroid the squared distance is summed over
// the features in index order and the running minimum kept (strict "<": lowest index on ties).
template <typename T>
__global__ __launch_bounds__(256) void naive_assign_kernel(const T *X, const T *C, int64_t N, int D, int K,
                                                           int32_t *labels, T *mindist)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= N) return;
    const T *x = X + i * D;
    T best = 0;
    int bj = 0;
    for (int j = 0; j < K; ++j) {
        const T *c = C + (int64_t)j * D;
        T s = 0;
        for (int d = 0; d < D; ++d) {
            const T diff = x[d] - c[d];
            s += diff * diff;
        }
        if (j == 0 || s < best) {
            best = s;
            bj = j;
        }
    }
    labels[i] = bj;
    if (mindist) mindist[i] = best;
}

// cn[j] = sum_d C[j][d]^2: one wave per centroid
template <typename T>
__global__ __launch_bounds__(256) void abl_norms_kernel(const T *C, int D, int K, T *cn)
{
    const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (j >= K) return;
    T s = 0;
    for (int d = lane; d < D; d += 64) s += C[(int64_t)j * D + d] * C[(int64_t)j * D + d];
    for (int m = 1; m < 64; m <<= 1) s += __shfl_xor(s, m, 64);
    if (lane == 0) cn[j] = s;
}

// Row i of S holds x_i . c_j for all j.  One wave per row: dist = ||x||^2 + ||c_j||^2 - 2 S_ij,
// of which only ||c_j||^2 - 2 S_ij takes part in the comparison; wave arg-min, lowest index
// on ties; ||x||^2 is added for the reported distance (clamped at zero).
template <typename T>
__global__ __launch_bounds__(256) void abl_rowmin_kernel(const T *S, const T *cn, const T *X, int64_t N, int D,
                                                         int K, int32_t *labels, T *mindist)
{
    const int64_t i = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (i >= N) return;
    const T *row = S + i * K;
    T best = 0;
    int bj = 0x7fffffff;
    for (int j = lane; j < K; j += 64) {
        const T v = cn[j] - 2 * row[j];
        if (bj == 0x7fffffff || v < best) {
            best = v;
            bj = j;
        }
    }
    for (int m = 1; m < 64; m <<= 1) {
        const T ob = __shfl_xor(best, m, 64);
        const int oj = __shfl_xor(bj, m, 64);
        if (oj != 0x7fffffff && (bj == 0x7fffffff || ob < best || (ob == best && oj < bj))) {
            best = ob;
            bj = oj;
        }
    }
    T xn = 0;
    if (mindist) {
        for (int d = lane; d < D; d += 64) xn += X[i * D + d] * X[i * D + d];
        for (int m = 1; m < 64; m <<= 1) xn += __shfl_xor(xn, m, 64);
    }
    if (lane == 0) {
        labels[i] = bj;
        if (mindist) {
            const T v = xn + best;
            mindist[i] = v > 0 ? v : 0;
        }
    }
}

rocblas_handle g_handle = nullptr;

bool check_shape(const void *X, const void *C, int64_t N, int32_t D, int32_t K, const int32_t *labels, int dtype)
{
    if (!X || !C || !labels || N < 1 || D < 1 || K < 1 || (dtype != 0 && dtype != 1) ||
        N > (int64_t)0x7fffffff * 4) {
        set_err("invalid argument (N=%lld D=%d K=%d dtype=%d)", (long long)N, D, K, dtype);
        return false;
    }
    return true;
}

}  // namespace

extern "C" {

const char *ftk_abl_last_error(void) { return g_err; }

int ftk_abl_naive_assign(int dtype, const void *X, const void *C, int64_t N, int32_t D, int32_t K,
                         int32_t *labels, void *mindist, void *hip_stream)
{
    if (!check_shape(X, C, N, D, K, labels, dtype)) return 1;
    hipStream_t st = (hipStream_t)hip_stream;
    const unsigned blocks = (unsigned)((N + 255) / 256);
    if (dtype == 0)
        hipLaunchKernelGGL(naive_assign_kernel<float>, dim3(blocks), dim3(256), 0, st, (const float *)X,
                           (const float *)C, N, D, K, labels, (float *)mindist);
    else
        hipLaunchKernelGGL(naive_assign_kernel<double>, dim3(blocks), dim3(256), 0, st, (const double *)X,
                           (const double *)C, N, D, K, labels, (double *)mindist);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_err("launch failed: %s", hipGetErrorString(e));
        return 4;
    }
    return 0;
}

size_t ftk_abl_gemm_workspace_bytes(int dtype, int64_t N, int32_t K)
{
    const size_t esz = dtype == 1 ? 8 : 4;
    if (N < 1 || K < 1) return 0;
    return ((size_t)N * (size_t)K + (size_t)K) * esz + 256;
}

int ftk_abl_gemm_assign(int dtype, const void *X, const void *C, int64_t N, int32_t D, int32_t K,
                        int32_t *labels, void *mindist, void *workspace, size_t workspace_bytes,
                        void *hip_stream)
{
    if (!check_shape(X, C, N, D, K, labels, dtype)) return 1;
    if (N > 0x7fffffff) {
        set_err("N=%lld exceeds the 32-bit extents of the vendor GEMM interface", (long long)N);
        return 1;
    }
    if (!workspace || workspace_bytes < ftk_abl_gemm_workspace_bytes(dtype, N, K)) {
        set_err("workspace too small: %zu < %zu", workspace_bytes, ftk_abl_gemm_workspace_bytes(dtype, N, K));
        return 3;
    }
    hipStream_t st = (hipStream_t)hip_stream;
    if (!g_handle && rocblas_create_handle(&g_handle) != rocblas_status_success) {
        g_handle = nullptr;
        set_err("rocblas_create_handle failed");
        return 4;
    }
    if (rocblas_set_stream(g_handle, st) != rocblas_status_success ||
        rocblas_set_pointer_mode(g_handle, rocblas_pointer_mode_host) != rocblas_status_success) {
        set_err("rocblas stream / pointer mode set-up failed");
        return 4;
    }
    const size_t esz = dtype == 1 ? 8 : 4;
    char *S = (char *)workspace;
    char *cn = S + (((size_t)N * (size_t)K * esz + 255) / 256) * 256;
    // Row-major S [N x K] = X C^T is, read column-major, the [K x N] matrix (C as [D x K])^T (X as [D x N]).
    rocblas_status rs;
    if (dtype == 0) {
        const float one = 1.f, zero = 0.f;
        hipLaunchKernelGGL(abl_norms_kernel<float>, dim3((K + 3) / 4), dim3(256), 0, st, (const float *)C, D, K,
                           (float *)cn);
        rs = rocblas_sgemm(g_handle, rocblas_operation_transpose, rocblas_operation_none, K, (rocblas_int)N, D, &one,
                           (const float *)C, D, (const float *)X, D, &zero, (float *)S, K);
        if (rs == rocblas_status_success)
            hipLaunchKernelGGL(abl_rowmin_kernel<float>, dim3((unsigned)((N + 3) / 4)), dim3(256), 0, st,
                               (const float *)S, (const float *)cn, (const float *)X, N, D, K, labels,
                               (float *)mindist);
    } else {
        const double one = 1.0, zero = 0.0;
        hipLaunchKernelGGL(abl_norms_kernel<double>, dim3((K + 3) / 4), dim3(256), 0, st, (const double *)C, D, K,
                           (double *)cn);
        rs = rocblas_dgemm(g_handle, rocblas_operation_transpose, rocblas_operation_none, K, (rocblas_int)N, D, &one,
                           (const double *)C, D, (const double *)X, D, &zero, (double *)S, K);
        if (rs == rocblas_status_success)
            hipLaunchKernelGGL(abl_rowmin_kernel<double>, dim3((unsigned)((N + 3) / 4)), dim3(256), 0, st,
                               (const double *)S, (const double *)cn, (const double *)X, N, D, K, labels,
                               (double *)mindist);
    }
    if (rs != rocblas_status_success) {
        set_err("rocBLAS gemm failed with status %d", (int)rs);
        return 4;
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_err("launch failed: %s", hipGetErrorString(e));
        return 4;
    }
    return 0;
}

}  // extern "C"
