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


// ---- Sections 3.1.3 / 3.1.4: the distance GEMM on the plain ALUs with the minimum fused in -------
// A workgroup of 256 threads owns a 128-point by 128-centroid tile of the product; a thread
// accumulates an 8 x 8 register block of it from operand tiles of 8 features staged in LDS
// (transposed, so that a thread's eight points / eight centroids are contiguous).  The epilogue
// forms cn_j - 2 S_ij, takes the minimum over the thread's eight centroids (thread level), then
// over the sixteen threads that share a point (threadblock level), and leaves ONE candidate per
// point and centroid block: the N x K product never reaches memory.
//   V2 (Section 3.1.3): the candidates go to a [N][K/128] array, a second kernel reduces each row.
//   V3 (Section 3.1.4): the candidates of all centroid blocks meet in one 64-bit word per point
//       through a device-wide atomic minimum on (value bits, index) - the counterpart of the
//       paper's per-row lock and broadcast - so the reduction kernel disappears (fp32 only: the
//       key packs a 32-bit value with the index).
constexpr int VB = 128, VK = 8;

// order-preserving map of a float onto unsigned integers (negative values included)
__device__ __forceinline__ unsigned ordered_bits(float v)
{
    const unsigned b = __float_as_uint(v);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float from_ordered_bits(unsigned o)
{
    return __uint_as_float((o & 0x80000000u) ? (o & 0x7fffffffu) : ~o);
}

template <typename T, bool ATOMIC>
__global__ __launch_bounds__(256) void abl_fused_alu_kernel(const T *X, const T *C, const T *cn, int64_t N, int D,
                                                            int K, T *part_val, int32_t *part_idx, int ncb,
                                                            unsigned long long *keys)
{
    __shared__ T Xs[VK][VB + 4], Cs[VK][VB + 4];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;            // centroid / point sub-blocks of 8
    const int64_t p0 = (int64_t)blockIdx.x * VB;
    const int j0 = blockIdx.y * VB;
    T acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = T(0);
    for (int d0 = 0; d0 < D; d0 += VK) {
        // 128 rows x 8 features of each operand: four elements per thread
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int idx = tid + 256 * e, row = idx >> 3, dd = idx & 7;
            const int64_t p = p0 + row;
            const int j = j0 + row;
            Xs[dd][row] = (p < N && d0 + dd < D) ? X[p * D + d0 + dd] : T(0);
            Cs[dd][row] = (j < K && d0 + dd < D) ? C[(int64_t)j * D + d0 + dd] : T(0);
        }
        __syncthreads();
#pragma unroll
        for (int dd = 0; dd < VK; ++dd) {
            T xv[8], cv[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) xv[i] = Xs[dd][ty * 8 + i];
#pragma unroll
            for (int j = 0; j < 8; ++j) cv[j] = Cs[dd][tx * 8 + j];
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[i][j] += xv[i] * cv[j];
        }
        __syncthreads();
    }
    T cnv[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) cnv[j] = (j0 + tx * 8 + j < K) ? cn[j0 + tx * 8 + j] : T(0);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        // thread level: the best of this thread's eight centroids (increasing index, strict "<")
        T best = 0;
        int bj = 0x7fffffff;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int jj = j0 + tx * 8 + j;
            const T v = cnv[j] - 2 * acc[i][j];
            if (jj < K && (bj == 0x7fffffff || v < best)) {
                best = v;
                bj = jj;
            }
        }
        // threadblock level: the sixteen threads of a point sit in sixteen consecutive lanes
#pragma unroll
        for (int m = 1; m < 16; m <<= 1) {
            const T ob = __shfl_xor(best, m, 64);
            const int oj = __shfl_xor(bj, m, 64);
            if (oj != 0x7fffffff && (bj == 0x7fffffff || ob < best || (ob == best && oj < bj))) {
                best = ob;
                bj = oj;
            }
        }
        const int64_t p = p0 + ty * 8 + i;
        if (tx == 0 && p < N && bj != 0x7fffffff) {
            if constexpr (ATOMIC) {
                const unsigned long long key = ((unsigned long long)ordered_bits((float)best) << 32) | (unsigned)bj;
                atomicMin(keys + p, key);
            } else {
                part_val[p * ncb + blockIdx.y] = best;
                part_idx[p * ncb + blockIdx.y] = bj;
            }
        }
    }
}

// V2: one thread per point reduces its K/128 candidates; V3: unpacks the key.  Both add ||x||^2.
template <typename T, bool ATOMIC>
__global__ __launch_bounds__(256) void abl_fused_finish_kernel(const T *X, int64_t N, int D, const T *part_val,
                                                               const int32_t *part_idx, int ncb,
                                                               const unsigned long long *keys, int32_t *labels,
                                                               T *mindist)
{
    const int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (p >= N) return;
    T best = 0;
    int bj = 0x7fffffff;
    if constexpr (ATOMIC) {
        const unsigned long long key = keys[p];
        bj = (int)(unsigned)(key & 0xffffffffu);
        best = (T)from_ordered_bits((unsigned)(key >> 32));
    } else {
        for (int b = 0; b < ncb; ++b) {  // increasing centroid index: strict "<" keeps the lowest on ties
            const T v = part_val[p * ncb + b];
            if (bj == 0x7fffffff || v < best) {
                best = v;
                bj = part_idx[p * ncb + b];
            }
        }
    }
    labels[p] = bj;
    if (mindist) {
        T xn = 0;
        for (int d = 0; d < D; ++d) xn += X[p * D + d] * X[p * D + d];
        const T v = xn + best;
        mindist[p] = v > 0 ? v : 0;
    }
}

__global__ void abl_fill_keys_kernel(unsigned long long *keys, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) keys[i] = ~0ull;
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

template <typename T>
int fused_alu_t(const void *X, const void *C, int64_t N, int32_t D, int32_t K, int32_t *labels, void *mindist,
                       int variant, char *ws, hipStream_t st)
{
    const size_t esz = sizeof(T);
    const int ncb = (K + VB - 1) / VB;
    T *cn = (T *)ws;
    char *rest = ws + ((size_t)K * esz + 255) / 256 * 256;
    hipLaunchKernelGGL((abl_norms_kernel<T>), dim3((K + 3) / 4), dim3(256), 0, st, (const T *)C, D, K, cn);
    dim3 grid((unsigned)((N + VB - 1) / VB), (unsigned)ncb);
    const unsigned fin = (unsigned)((N + 255) / 256);
    if (variant == 3) {
        unsigned long long *keys = (unsigned long long *)rest;
        hipLaunchKernelGGL(abl_fill_keys_kernel, dim3(fin), dim3(256), 0, st, keys, N);
        hipLaunchKernelGGL((abl_fused_alu_kernel<T, true>), grid, dim3(256), 0, st, (const T *)X, (const T *)C, cn, N, D,
                           K, (T *)nullptr, (int32_t *)nullptr, ncb, keys);
        hipLaunchKernelGGL((abl_fused_finish_kernel<T, true>), dim3(fin), dim3(256), 0, st, (const T *)X, N, D,
                           (const T *)nullptr, (const int32_t *)nullptr, ncb, keys, labels, (T *)mindist);
    } else {
        T *pv = (T *)rest;
        int32_t *pi = (int32_t *)(rest + ((size_t)N * ncb * esz + 255) / 256 * 256);
        hipLaunchKernelGGL((abl_fused_alu_kernel<T, false>), grid, dim3(256), 0, st, (const T *)X, (const T *)C, cn, N,
                           D, K, pv, pi, ncb, (unsigned long long *)nullptr);
        hipLaunchKernelGGL((abl_fused_finish_kernel<T, false>), dim3(fin), dim3(256), 0, st, (const T *)X, N, D, pv, pi,
                           ncb, (const unsigned long long *)nullptr, labels, (T *)mindist);
    }
    if (hipGetLastError() != hipSuccess) {
        set_err("kernel launch failed");
        return 4;
    }
    return 0;
}

// One v_mfma_f32_32x32x16_bf16 per wave on operands given as plain matrices: D = A B + C with A
// [32][16] and B [16][32] in bf16 (bit patterns) and C, D [32][32] in fp32, `tiles` independent
// problems.  Lane l supplies A[l % 32][8 (l / 32) .. + 7] and B[8 (l / 32) .. + 7][l % 32]; its
// register r holds D[8 (r / 4) + 4 (l / 32) + r % 4][l % 32].  Exists so that a test can hold the
// instruction's rounding behaviour - which the fast assignment's error bound is built on and no
// document states - against the exact sums.
typedef __bf16 abl_bf16x8 __attribute__((ext_vector_type(8)));
typedef float abl_floatx16 __attribute__((ext_vector_type(16)));
__global__ __launch_bounds__(64) void abl_mfma_bf16_kernel(const uint16_t *A, const uint16_t *B, const float *C, float *Dout)
{
    const int lane = threadIdx.x, col = lane & 31, g = lane >> 5;
    const size_t t = blockIdx.x;
    const uint16_t *a = A + t * 32 * 16, *b = B + t * 16 * 32;
    const float *c = C + t * 32 * 32;
    float *d = Dout + t * 32 * 32;
    abl_bf16x8 av, bv;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        av[e] = __builtin_bit_cast(__bf16, a[col * 16 + 8 * g + e]);
        bv[e] = __builtin_bit_cast(__bf16, b[(8 * g + e) * 32 + col]);
    }
    abl_floatx16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = c[(8 * (r / 4) + 4 * g + r % 4) * 32 + col];
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc, 0, 0, 0);
#pragma unroll
    for (int r = 0; r < 16; ++r) d[(8 * (r / 4) + 4 * g + r % 4) * 32 + col] = acc[r];
}


// The fp32 and fp64 instructions of the main path, the same way: v_mfma_f32_32x32x2_f32 (A [32][2],
// B [2][32], C and D [32][32]; lane l supplies A[l % 32][l / 32] and B[l / 32][l % 32]) and
// v_mfma_f64_16x16x4_f64 (A [16][4], B [4][16], C and D [16][16]; lane l supplies A[l % 16][l / 16]
// and B[l / 16][l % 16], register r holds D[4 r + l / 16][l % 16]).
__global__ __launch_bounds__(64) void abl_mfma_f32_kernel(const float *A, const float *B, const float *C, float *Dout)
{
    const int lane = threadIdx.x, col = lane & 31, g = lane >> 5;
    const size_t t = blockIdx.x;
    const float *c = C + t * 32 * 32;
    float *d = Dout + t * 32 * 32;
    abl_floatx16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = c[(8 * (r / 4) + 4 * g + r % 4) * 32 + col];
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(A[t * 64 + col * 2 + g], B[t * 64 + g * 32 + col], acc, 0, 0, 0);
#pragma unroll
    for (int r = 0; r < 16; ++r) d[(8 * (r / 4) + 4 * g + r % 4) * 32 + col] = acc[r];
}

typedef double abl_doublex4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(64) void abl_mfma_f64_kernel(const double *A, const double *B, const double *C, double *Dout)
{
    const int lane = threadIdx.x, col = lane & 15, g = lane >> 4;
    const size_t t = blockIdx.x;
    const double *c = C + t * 16 * 16;
    double *d = Dout + t * 16 * 16;
    abl_doublex4 acc;
#pragma unroll
    for (int r = 0; r < 4; ++r) acc[r] = c[(4 * r + g) * 16 + col];
    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(A[t * 64 + col * 4 + g], B[t * 64 + g * 16 + col], acc, 0, 0, 0);
#pragma unroll
    for (int r = 0; r < 4; ++r) d[(4 * r + g) * 16 + col] = acc[r];
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


size_t ftk_abl_fused_alu_workspace_bytes(int dtype, int64_t N, int32_t K, int32_t variant)
{
    const size_t esz = dtype == 0 ? 4 : 8;
    const size_t ncb = (size_t)(K + VB - 1) / VB;
    const size_t cn = ((size_t)K * esz + 255) / 256 * 256;
    if (variant == 3) return cn + (size_t)N * 8;
    return cn + (((size_t)N * ncb * esz + 255) / 256 * 256) + (size_t)N * ncb * 4;
}

int ftk_abl_fused_alu_assign(int dtype, const void *X, const void *C, int64_t N, int32_t D, int32_t K,
                             int32_t *labels, void *mindist, int32_t variant, void *workspace,
                             size_t workspace_bytes, void *hip_stream)
{
    if (!check_shape(X, C, N, D, K, labels, dtype)) return 1;
    if ((variant != 2 && variant != 3) || (variant == 3 && dtype != 0)) {
        set_err("invalid argument: variant %d (2 for both dtypes, 3 for fp32 only)", variant);
        return 1;
    }
    if (!workspace || workspace_bytes < ftk_abl_fused_alu_workspace_bytes(dtype, N, K, variant)) {
        set_err("workspace too small");
        return 3;
    }
    hipStream_t st = (hipStream_t)hip_stream;
    return dtype == 0 ? fused_alu_t<float>(X, C, N, D, K, labels, mindist, variant, (char *)workspace, st)
                      : fused_alu_t<double>(X, C, N, D, K, labels, mindist, variant, (char *)workspace, st);
}

int ftk_abl_mfma_bf16(const uint16_t *A, const uint16_t *B, const float *C, float *D, int32_t tiles, void *hip_stream)
{
    if (!A || !B || !C || !D || tiles <= 0) {
        set_err("invalid argument");
        return 1;
    }
    hipLaunchKernelGGL(abl_mfma_bf16_kernel, dim3((unsigned)tiles), dim3(64), 0, (hipStream_t)hip_stream, A, B, C, D);
    if (hipGetLastError() != hipSuccess) {
        set_err("kernel launch failed");
        return 4;
    }
    return 0;
}

int ftk_abl_mfma_f32(const float *A, const float *B, const float *C, float *D, int32_t tiles, void *hip_stream)
{
    if (!A || !B || !C || !D || tiles <= 0) {
        set_err("invalid argument");
        return 1;
    }
    hipLaunchKernelGGL(abl_mfma_f32_kernel, dim3((unsigned)tiles), dim3(64), 0, (hipStream_t)hip_stream, A, B, C, D);
    if (hipGetLastError() != hipSuccess) {
        set_err("kernel launch failed");
        return 4;
    }
    return 0;
}

int ftk_abl_mfma_f64(const double *A, const double *B, const double *C, double *D, int32_t tiles, void *hip_stream)
{
    if (!A || !B || !C || !D || tiles <= 0) {
        set_err("invalid argument");
        return 1;
    }
    hipLaunchKernelGGL(abl_mfma_f64_kernel, dim3((unsigned)tiles), dim3(64), 0, (hipStream_t)hip_stream, A, B, C, D);
    if (hipGetLastError() != hipSuccess) {
        set_err("kernel launch failed");
        return 4;
    }
    return 0;
}

}  // extern "C"
