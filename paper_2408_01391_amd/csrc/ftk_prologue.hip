// Small helper kernels around the assignment step: centroid norms (the "simple kernels" of
// Section 3.1.2), per-tile checksum rows of the centroid operand (the Y e1 / Y e2 encodings
// of Section 4.1), |x| maximum, row gather for the initial centroids, and a fixed-order sum.
#include "ftk_internal.h"
#include "ftk_mma.h"

namespace ftk {

__global__ void reset_assign_state_kernel(double *scal, int32_t *wl_count)
{
    if (threadIdx.x == 0) {
        scal[0] = 0.0;
        scal[1] = 0.0;    // largest truncation norm of a checksum row (two-piece fast path)
        wl_count[0] = 0;  // refine work-list length
        wl_count[1] = 0;  // dynamic point-block counter of the persistent small-D kernel
    }
}

// hcn[j] = ||c_j||^2 / 2 (accumulated in double) for j < Kpad, zero (or +inf) for the padding
// rows; scal[0] = max_j ||c_j||^2 via an integer max on the bit pattern (valid for non-negative
// doubles).  L = 2^lpr_log2 lanes share a row (one lane per row for short rows), and a wave
// issues ONE atomic for all its rows: with one atomic per row the kernel time was the
// serialised atomics on that single address.
//
// SINGLE: the whole job in one workgroup of 1024 threads, which then also resets the per-call
// state (plain stores instead of the reset kernel plus atomics) - one launch less for the
// common case of a small centroid matrix (up to 64K elements).
template <typename T, bool SINGLE>
__global__ __launch_bounds__(SINGLE ? 1024 : 256) void centroid_norms_kernel(const T *C, int D, int K, int Kpad,
                                                                            T *hcn, double *scal, int pad_inf,
                                                                            int lpr_log2, int32_t *wl_count)
{
    const int lane = threadIdx.x & 63;
    const int L = 1 << lpr_log2;
    const int rpw = 64 >> lpr_log2;  // rows per wave and step
    const int sub = lane & (L - 1);
    const int wave0 = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int nwaves = (int)(blockDim.x >> 6);  // SINGLE: the workgroup strides over all rows
    double m = 0.0;
    for (int wave = wave0; wave * rpw < Kpad; wave = SINGLE ? wave + nwaves : Kpad) {
        const int j = wave * rpw + (lane >> lpr_log2);
        double s = 0.0;
        if (j < K) {
            const T *c = C + (int64_t)j * D;
            // several loads in flight per lane: the job is a latency chain otherwise
#pragma unroll 8
            for (int d = sub; d < D; d += L) {
                const double v = (double)c[d];
                s = fma(v, v, s);
            }
        }
        for (int mask = L >> 1; mask >= 1; mask >>= 1) s += __shfl_xor(s, mask, 64);
        if (sub == 0 && j < Kpad) hcn[j] = (j >= K && pad_inf) ? (T)__builtin_huge_val() : (T)(0.5 * s);
        m = s > m ? s : m;  // s is zero for rows at or beyond K
    }
#pragma unroll
    for (int mask = 32; mask >= 1; mask >>= 1) {
        const double o = __shfl_xor(m, mask, 64);
        m = o > m ? o : m;
    }
    if constexpr (SINGLE) {
        __shared__ double sh_m[16];
        if (lane == 0) sh_m[threadIdx.x >> 6] = m;
        __syncthreads();
        if (threadIdx.x == 0) {
            for (int i = 1; i < (int)(blockDim.x >> 6); ++i) m = sh_m[i] > m ? sh_m[i] : m;
            scal[0] = m;
            scal[1] = 0.0;    // largest truncation norm of a checksum row (two-piece fast path)
            wl_count[0] = 0;  // refine work-list length
            wl_count[1] = 0;  // dynamic point-block counter of the persistent small-D kernel
        }
    } else {
        if (lane == 0 && m > 0.0)
            atomicMax((unsigned long long *)scal, (unsigned long long)__double_as_longlong(m));
    }
}

// Checksum rows of one centroid tile (TM consecutive centroids, TM <= 1024):
//   v1[d] = sum_r c_{r,d}            (weights e1 = 1)
//   v2[d] = sum_r (r+1) c_{r,d}      (weights e2 = 1..TM)
// in double, rounded once, and the matching sums of the (rounded) half norms, kept in double.  A workgroup covers 64
// features of one tile: 16 thread groups each add every 16th row (coalesced 64-element reads),
// the partial sums are combined in LDS in a fixed order.
template <typename T>
__global__ __launch_bounds__(1024) void centroid_checksum_kernel(const T *C, const T *hcn, int D, int D8,
                                                                 int K, int TM, T *v1, T *v2, double *cs)
{
    __shared__ double sh1[16][64], sh2[16][64];
    const int tile = blockIdx.x;
    const int j0 = tile * TM;
    const int dl = threadIdx.x & 63, rg = threadIdx.x >> 6;
    const int d = blockIdx.y * 64 + dl;
    double s1 = 0.0, s2 = 0.0;
    if (d < D) {
        for (int r = rg; r < TM && j0 + r < K; r += 16) {
            const double v = (double)C[(int64_t)(j0 + r) * D + d];
            s1 += v;
            s2 = fma((double)(r + 1), v, s2);
        }
    }
    sh1[rg][dl] = s1;
    sh2[rg][dl] = s2;
    __syncthreads();
    if (rg == 0 && d < D8) {
        for (int g2 = 1; g2 < 16; ++g2) {
            s1 += sh1[g2][dl];
            s2 += sh2[g2][dl];
        }
        v1[(int64_t)tile * D8 + d] = (T)s1;
        v2[(int64_t)tile * D8 + d] = (T)s2;
    }
    if (blockIdx.y == 0) {
        __syncthreads();
        double *f1 = &sh1[0][0], *f2 = &sh2[0][0];  // 1024 slots each
        const int r = threadIdx.x;
        const double h = (r < TM && j0 + r < K) ? (double)hcn[j0 + r] : 0.0;
        f1[r] = h;
        f2[r] = (double)(r + 1) * h;
        __syncthreads();
        for (int half = 512; half >= 1; half >>= 1) {
            if (r < half) {
                f1[r] += f1[r + half];
                f2[r] += f2[r + half];
            }
            __syncthreads();
        }
        if (r == 0) {
            cs[2 * tile] = f1[0];
            cs[2 * tile + 1] = f2[0];
        }
    }
}

ftk_status launch_centroid_prologue(const AssignCall &c, const AssignPlan &p, const Workspace &w,
                                    hipStream_t st)
{
    const int Kpad = p.nkc * p.KC;
    if ((size_t)Kpad > w.hcn_entries) {
        set_error("internal: plan pads K=%d to %d rows, workspace reserves %zu", c.K, Kpad, w.hcn_entries);
        return FTK_EWORKSPACE;
    }
    // lanes per row: 1 for rows up to 32 features, 8 up to 256, else the whole wave
    const int lpr_log2 = c.D <= 32 ? 0 : (c.D <= 256 ? 3 : 6);
    const bool single = (int64_t)Kpad * c.D <= 65536;
    const int blocks = single ? 1 : (int)ceil_div(Kpad, 4 * (64 >> lpr_log2));
    const int threads = single ? 1024 : 256;
    if (!single) hipLaunchKernelGGL(reset_assign_state_kernel, dim3(1), dim3(64), 0, st, w.scal, w.wl_count);
    const int ntiles = p.nkc;  // generic variant: one checksum row pair per K-chunk
    const bool generic_ft = c.ft != FTK_FT_OFF && p.variant == VAR_GENERIC;
    if (c.dtype == FTK_F32) {
        if (single)
            hipLaunchKernelGGL((centroid_norms_kernel<float, true>), dim3(blocks), dim3(threads), 0, st,
                               (const float *)c.C, c.D, c.K, Kpad, (float *)w.hcn, w.scal, (int)p.hcn_pad_inf,
                               lpr_log2, w.wl_count);
        else
            hipLaunchKernelGGL((centroid_norms_kernel<float, false>), dim3(blocks), dim3(threads), 0, st,
                               (const float *)c.C, c.D, c.K, Kpad, (float *)w.hcn, w.scal, (int)p.hcn_pad_inf,
                               lpr_log2, w.wl_count);
        if (generic_ft)
            hipLaunchKernelGGL((centroid_checksum_kernel<float>), dim3(ntiles, (unsigned)ceil_div(p.D8, 64)), dim3(1024), 0, st,
                               (const float *)c.C, (const float *)w.hcn, c.D, p.D8, c.K, p.KC,
                               (float *)w.chk_v1, (float *)w.chk_v2, w.chk_sd);
    } else {
        if (single)
            hipLaunchKernelGGL((centroid_norms_kernel<double, true>), dim3(blocks), dim3(threads), 0, st,
                               (const double *)c.C, c.D, c.K, Kpad, (double *)w.hcn, w.scal, (int)p.hcn_pad_inf,
                               lpr_log2, w.wl_count);
        else
            hipLaunchKernelGGL((centroid_norms_kernel<double, false>), dim3(blocks), dim3(threads), 0, st,
                               (const double *)c.C, c.D, c.K, Kpad, (double *)w.hcn, w.scal, (int)p.hcn_pad_inf,
                               lpr_log2, w.wl_count);
        if (generic_ft)
            hipLaunchKernelGGL((centroid_checksum_kernel<double>), dim3(ntiles, (unsigned)ceil_div(p.D8, 64)), dim3(1024), 0, st,
                               (const double *)c.C, (const double *)w.hcn, c.D, p.D8, c.K, p.KC,
                               (double *)w.chk_v1, (double *)w.chk_v2, w.chk_sd);
    }
    if (c.ft != FTK_FT_OFF && p.variant != VAR_GENERIC) FTK_TRY(launch_smalld_checksums(c, p, w, st));
    FTK_TRY_HIP(hipGetLastError());
    return FTK_OK;
}

__global__ void zero_ints_kernel(int32_t *p, int n)
{
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) p[i] = 0;
}

ftk_status launch_zero_ints(int32_t *p, int n, hipStream_t st)
{
    hipLaunchKernelGGL(zero_ints_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, st, p, n);
    FTK_TRY_HIP(hipGetLastError());
    return FTK_OK;
}

// ---- |x| maximum ---------------------------------------------------------------------------
__global__ void reset_double_kernel(double *p)
{
    if (threadIdx.x == 0) p[0] = 0.0;
}

template <typename T>
__global__ __launch_bounds__(256) void absmax_kernel(const T *X, int64_t count, double *out)
{
    double m = 0.0;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride) {
        const double v = fabs((double)X[i]);
        m = (v > m && v < __builtin_huge_val()) ? v : m;  // NaN and Inf never raise the maximum
    }
#pragma unroll
    for (int mask = 32; mask >= 1; mask >>= 1) {
        const double o = __shfl_xor(m, mask, 64);
        m = o > m ? o : m;
    }
    if ((threadIdx.x & 63) == 0 && m > 0.0)
        atomicMax((unsigned long long *)out, (unsigned long long)__double_as_longlong(m));
}

// 16-byte vectorised variant for aligned, large inputs
template <typename T>
__global__ __launch_bounds__(256) void absmax_vec_kernel(const T *X, int64_t nvec, double *out)
{
    using F = typename Mma<T>::frag_t;
    constexpr int E = Mma<T>::E;
    const F *Xv = reinterpret_cast<const F *>(X);
    T m = T(0);
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += stride) {
        const F f = Xv[i];
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const T v = fabs(f[e]);
            m = (v > m && v < Mma<T>::huge()) ? v : m;  // NaN and Inf never raise the maximum
        }
    }
    double md = (double)m;
#pragma unroll
    for (int mask = 32; mask >= 1; mask >>= 1) {
        const double o = __shfl_xor(md, mask, 64);
        md = o > md ? o : md;
    }
    if ((threadIdx.x & 63) == 0 && md > 0.0)
        atomicMax((unsigned long long *)out, (unsigned long long)__double_as_longlong(md));
}

ftk_status launch_absmax(ftk_dtype dtype, const void *X, int64_t count, double *out, hipStream_t st)
{
    hipLaunchKernelGGL(reset_double_kernel, dim3(1), dim3(64), 0, st, out);
    const int E = dtype == FTK_F32 ? 4 : 2;
    const size_t esz = dtype == FTK_F32 ? 4 : 8;
    int64_t nvec = ((uintptr_t)X % 16 == 0) ? count / E : 0;
    if (nvec > 0) {
        const int blocks = (int)(ceil_div(nvec, 256) < 2048 ? ceil_div(nvec, 256) : 2048);
        if (dtype == FTK_F32)
            hipLaunchKernelGGL((absmax_vec_kernel<float>), dim3(blocks), dim3(256), 0, st,
                               (const float *)X, nvec, out);
        else
            hipLaunchKernelGGL((absmax_vec_kernel<double>), dim3(blocks), dim3(256), 0, st,
                               (const double *)X, nvec, out);
    }
    const int64_t done = nvec * E;
    if (done < count) {
        const int64_t rest = count - done;
        const int blocks = (int)(ceil_div(rest, 256) < 1024 ? ceil_div(rest, 256) : 1024);
        const char *tail = (const char *)X + done * esz;
        if (dtype == FTK_F32)
            hipLaunchKernelGGL((absmax_kernel<float>), dim3(blocks), dim3(256), 0, st,
                               (const float *)tail, rest, out);
        else
            hipLaunchKernelGGL((absmax_kernel<double>), dim3(blocks), dim3(256), 0, st,
                               (const double *)tail, rest, out);
    }
    FTK_TRY_HIP(hipGetLastError());
    return FTK_OK;
}

// ---- initial centroids: C[k] = X[idx[k]] ------------------------------------------------
template <typename T>
__global__ void gather_rows_kernel(const T *X, int D, const int64_t *idx, int K, T *C)
{
    const int k = blockIdx.x;
    if (k >= K) return;
    const T *src = X + idx[k] * D;
    for (int d = threadIdx.x; d < D; d += blockDim.x) C[(int64_t)k * D + d] = src[d];
}

ftk_status launch_gather_rows(ftk_dtype dtype, const void *X, int D, const int64_t *idx_dev, int K,
                              void *C, hipStream_t st)
{
    if (dtype == FTK_F32)
        hipLaunchKernelGGL((gather_rows_kernel<float>), dim3(K), dim3(64), 0, st, (const float *)X, D,
                           idx_dev, K, (float *)C);
    else
        hipLaunchKernelGGL((gather_rows_kernel<double>), dim3(K), dim3(64), 0, st, (const double *)X,
                           D, idx_dev, K, (double *)C);
    FTK_TRY_HIP(hipGetLastError());
    return FTK_OK;
}

// ---- objective: sum of a vector in double, fixed order (block partials, then one block) ----
constexpr int SUM_BLOCKS = 512;

template <typename T>
__global__ __launch_bounds__(256) void sum_partials_kernel(const T *v, int64_t n, double *partials)
{
    __shared__ double sh[256];
    const int64_t per = (n + gridDim.x - 1) / gridDim.x;
    const int64_t lo = per * blockIdx.x;
    const int64_t hi = lo + per < n ? lo + per : n;
    double s = 0.0;
    for (int64_t i = lo + threadIdx.x; i < hi; i += 256) s += (double)v[i];
    sh[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w >= 1; w >>= 1) {
        if ((int)threadIdx.x < w) sh[threadIdx.x] += sh[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) partials[blockIdx.x] = sh[0];
}

__global__ __launch_bounds__(256) void sum_final_kernel(const double *partials, int n, double *out)
{
    __shared__ double sh[256];
    double s = 0.0;
    for (int i = threadIdx.x; i < n; i += 256) s += partials[i];
    sh[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w >= 1; w >>= 1) {
        if ((int)threadIdx.x < w) sh[threadIdx.x] += sh[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[0] = sh[0];
}

ftk_status launch_sum_to_double(ftk_dtype dtype, const void *v, int64_t n, double *partials,
                                double *out, hipStream_t st)
{
    if (dtype == FTK_F32)
        hipLaunchKernelGGL((sum_partials_kernel<float>), dim3(SUM_BLOCKS), dim3(256), 0, st,
                           (const float *)v, n, partials);
    else
        hipLaunchKernelGGL((sum_partials_kernel<double>), dim3(SUM_BLOCKS), dim3(256), 0, st,
                           (const double *)v, n, partials);
    hipLaunchKernelGGL(sum_final_kernel, dim3(1), dim3(256), 0, st, partials, SUM_BLOCKS, out);
    FTK_TRY_HIP(hipGetLastError());
    return FTK_OK;
}

}  // namespace ftk
