// Centroid update, Eq. (2): per-cluster sums and counts, then the averaging pass.
//
// The paper's kernel (Section 3.1.2) has every thread add its point into the global sums with
// floating-point atomics, whose result depends on the order in which the adds land.  Here the
// sums are accumulated in 64-bit FIXED POINT: every coordinate is scaled by a power of two
// fixed from max|x| and N so that no sum can overflow, rounded once to an integer, and added
// with integer atomics.  Integer addition is associative, so the sums - and the centroids -
// are bitwise identical from run to run whatever the schedule, and the only rounding is the
// one quantisation per coordinate (<= 2^-(62 - ceil(log2 N)) relative to max|x|).
//
// Accumulation is privatised in LDS: a workgroup owns a block of points and a [Ks x Ds] slice
// of the sum matrix that fits 64 KB, adds into it with LDS atomics, and flushes the non-zero
// cells to the global matrix with one integer atomic each.  Feature slices partition the
// columns of X and cluster slices partition its rows by label, so X is read once overall.
#include "ftk_internal.h"
#include "ftk_mma.h"

namespace ftk {

constexpr int UPD_CELLS = 8192;  // int64 cells per workgroup slice (64 KB)
constexpr int UPD_TARGET_WGS = 512;

struct UpdatePlan {
    int Ks, Ds, nks, nds, tx_log2;
    int64_t rows_per_chunk;
    int chunks;
    bool aligned;
};

static UpdatePlan plan_update(ftk_dtype dtype, const void *X, int64_t N, int D, int K)
{
    UpdatePlan u;
    const int E = dtype == FTK_F32 ? 4 : 2;
    u.aligned = (D % E == 0) && ((uintptr_t)X % 16 == 0);
    const int line = dtype == FTK_F32 ? 32 : 16;  // features per 128-byte line
    if ((int64_t)K * D <= UPD_CELLS) {
        u.Ks = K;
        u.Ds = D;
    } else {
        int ds = UPD_CELLS / K;          // widest feature slice with all clusters resident
        if (ds < line) ds = line;        // never read less than one line per row
        if (ds > D) ds = D;
        if (u.aligned) ds = ds / E * E;
        if (ds < 1) ds = 1;
        u.Ds = ds;
        int ks = UPD_CELLS / ds;
        u.Ks = ks < K ? (ks < 1 ? 1 : ks) : K;
    }
    u.nds = (int)ceil_div(D, u.Ds);
    u.nks = (int)ceil_div(K, u.Ks);
    const int slices = u.nds * u.nks;
    int chunks = UPD_TARGET_WGS / slices;
    if (chunks < 1) chunks = 1;
    if (chunks > ceil_div(N, 256)) chunks = (int)ceil_div(N, 256);
    u.chunks = chunks;
    u.rows_per_chunk = ceil_div(N, chunks);
    const int ppr = u.aligned ? (u.Ds + E - 1) / E : u.Ds;  // pieces per row slice
    int l2 = 0;
    while ((1 << l2) < ppr && l2 < 8) ++l2;
    u.tx_log2 = l2;
    return u;
}

__global__ void update_zero_kernel(unsigned long long *sums, int64_t n, int32_t *counts, int K)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) sums[i] = 0ull;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < K; i += stride) counts[i] = 0;
}

// scale = 2^(62 - ceil(log2 N) - (ilogb(absmax) + 1)): N * max|x| * scale <= 2^62
__device__ __forceinline__ double fixed_point_scale(double absmax, int64_t N)
{
    int L = 0;
    while (((int64_t)1 << L) < N) ++L;
    if (!(absmax > 0.0) || !(absmax < __builtin_huge_val())) return 1.0;
    return ldexp(1.0, 62 - L - (ilogb(absmax) + 1));
}

template <typename T, bool ALIGNED>
__global__ __launch_bounds__(256) void update_accumulate_kernel(
    const T *X, const int32_t *labels, int64_t N, int D, int K, const double *absmax_p,
    unsigned long long *sums, int32_t *counts, int Ks, int Ds, int nds, int tx_log2,
    int64_t rows_per_chunk)
{
    using F = typename Mma<T>::frag_t;
    constexpr int E = ALIGNED ? Mma<T>::E : 1;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    unsigned long long *cell = reinterpret_cast<unsigned long long *>(lds_raw);
    int *cnt = reinterpret_cast<int *>(cell + (size_t)Ks * Ds);

    const int tid = threadIdx.x;
    const int slice = blockIdx.y;
    const int ds_i = slice % nds, ks_i = slice / nds;
    const int d0 = ds_i * Ds, k0 = ks_i * Ks;
    const int dn = min(Ds, D - d0);  // features in this slice
    const int kn = min(Ks, K - k0);
    for (int i = tid; i < Ks * Ds; i += 256) cell[i] = 0ull;
    for (int i = tid; i < Ks; i += 256) cnt[i] = 0;
    __syncthreads();

    const double scale = fixed_point_scale(*absmax_p, N);
    const int TX = 1 << tx_log2, TY = 256 >> tx_log2;
    const int tx = tid & (TX - 1), ty = tid >> tx_log2;
    const int ppr = (dn + E - 1) / E;
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_chunk;
    const int64_t r1 = r0 + rows_per_chunk < N ? r0 + rows_per_chunk : N;

    for (int64_t row = r0 + ty; row < r1; row += TY) {
        const int lab = labels[row] - k0;
        if ((unsigned)lab >= (unsigned)kn) continue;
        if (tx == 0 && ds_i == 0) atomicAdd(&cnt[lab], 1);
        const T *xr = X + row * D + d0;
        unsigned long long *dst = cell + (size_t)lab * Ds;
        for (int pc = tx; pc < ppr; pc += TX) {
            if constexpr (ALIGNED) {
                const F f = *reinterpret_cast<const F *>(xr + pc * E);
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    const long long q = __double2ll_rn((double)f[e] * scale);
                    atomicAdd(dst + pc * E + e, (unsigned long long)q);
                }
            } else {
                const long long q = __double2ll_rn((double)xr[pc] * scale);
                atomicAdd(dst + pc, (unsigned long long)q);
            }
        }
    }
    __syncthreads();
    for (int i = tid; i < kn * Ds; i += 256) {
        const int k = i / Ds, d = i - k * Ds;
        const unsigned long long v = cell[i];
        if (v != 0ull && d < dn) atomicAdd(sums + (int64_t)(k0 + k) * D + d0 + d, v);
    }
    if (ds_i == 0)
        for (int i = tid; i < kn; i += 256)
            if (cnt[i]) atomicAdd(counts + k0 + i, cnt[i]);
}

// Averaging pass ("the last kernel", Section 3.1.1): C_j = sum_j / count_j, rounded once;
// a cluster without points keeps its previous centroid.
template <typename T>
__global__ __launch_bounds__(256) void update_finalize_kernel(const unsigned long long *sums,
                                                              const int32_t *counts, int64_t N, int D,
                                                              int K, const double *absmax_p, T *C)
{
    const double inv = 1.0 / fixed_point_scale(*absmax_p, N);
    const int64_t n = (int64_t)K * D;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const int c = counts[i / D];
        if (c > 0) C[i] = (T)(((double)(long long)sums[i] * inv) / (double)c);
    }
}

ftk_status launch_update(ftk_dtype dtype, const void *X, const int32_t *labels, int64_t N, int D,
                         int K, void *C, int32_t *counts, const double *absmax, const Workspace &w,
                         hipStream_t st)
{
    const UpdatePlan u = plan_update(dtype, X, N, D, K);
    const int64_t cells = (int64_t)K * D;
    unsigned long long *sums = reinterpret_cast<unsigned long long *>(w.fx_sums);
    {
        const int blocks = (int)(ceil_div(cells, 256) < 1024 ? ceil_div(cells, 256) : 1024);
        hipLaunchKernelGGL(update_zero_kernel, dim3(blocks), dim3(256), 0, st, sums, cells, counts, K);
    }
    const size_t lds = (size_t)u.Ks * u.Ds * 8 + (size_t)u.Ks * 4;
    dim3 grid(u.chunks, u.nds * u.nks), block(256);
#define FTK_LAUNCH_ACC(T, AL)                                                                      \
    hipLaunchKernelGGL((update_accumulate_kernel<T, AL>), grid, block, lds, st, (const T *)X, labels, \
                       N, D, K, absmax, sums, counts, u.Ks, u.Ds, u.nds, u.tx_log2, u.rows_per_chunk)
    if (dtype == FTK_F32) {
        if (u.aligned) FTK_LAUNCH_ACC(float, true);
        else FTK_LAUNCH_ACC(float, false);
    } else {
        if (u.aligned) FTK_LAUNCH_ACC(double, true);
        else FTK_LAUNCH_ACC(double, false);
    }
#undef FTK_LAUNCH_ACC
    {
        const int blocks = (int)(ceil_div(cells, 256) < 1024 ? ceil_div(cells, 256) : 1024);
        if (dtype == FTK_F32)
            hipLaunchKernelGGL((update_finalize_kernel<float>), dim3(blocks), dim3(256), 0, st, sums,
                               counts, N, D, K, absmax, (float *)C);
        else
            hipLaunchKernelGGL((update_finalize_kernel<double>), dim3(blocks), dim3(256), 0, st, sums,
                               counts, N, D, K, absmax, (double *)C);
    }
    FTK_TRY_HIP(hipGetLastError());
    return FTK_OK;
}

}  // namespace ftk
