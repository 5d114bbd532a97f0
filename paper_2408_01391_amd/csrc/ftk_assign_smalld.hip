// Small-D assignment kernel (fp32, D <= 32, rows 16-byte aligned).
//
// With few features the contraction per output tile is only D/2 matrix instructions, so the
// per-element epilogue work, not the matrix pipe, decides the speed (the paper notes the same
// for small feature counts in Section 5.1: data movement and the row-wise reduction become the
// critical part).  This variant therefore
//   * keeps the point fragments (B operand) in registers for the whole sweep over K: X is read
//     once, straight from HBM with 16-byte coalesced loads, and never goes through LDS;
//   * stages centroids (A operand) in LDS together with their -||c||^2/2 terms laid out in
//     accumulator order, so each tile starts from four broadcast 16-byte LDS reads;
//   * reduces every 32x32 output tile to ONE maximum per lane with v_max3 (half an op per
//     score) and keeps only the best three tile maxima and the two best tile numbers;
//   * after the sweep re-evaluates the (at most two) candidate groups of 16 centroids per lane
//     in direct-difference form, which yields the exact arg-min, resolves every near-tie the
//     cancelling expanded form cannot order, and gives an accurate minimum distance.
// A lane whose third-best tile maximum is still inside the rounding bound queues its point
// for the refine kernel.
#include <type_traits>

#include "ftk_internal.h"
#include "ftk_mma.h"

namespace ftk {

struct SmallArgs {
    const float *X;
    const float *C;
    const float *hcn;    // half squared norms, +inf beyond K, padded to nch*kch
    const double *scal;  // scal[0] = max_j ||c_j||^2
    int64_t N;
    int D, K;
    int kch;      // centroids per LDS chunk (multiple of 32)
    int nch;      // chunks
    int nblocks;  // point blocks (256*PT points each)
    int32_t *labels;
    float *mindist;
    int32_t *wl;
    int32_t *wl_count;
    ftk_ft_stats *stats;
    double band_coef;
};

__device__ __forceinline__ float max3f(float a, float b, float c) { return __builtin_fmaxf(__builtin_fmaxf(a, b), c); }

// Exact (direct-difference, fp32) distances of one point to the 16 centroids that lane group g
// owns in tile T; keeps the running (distance, index) minimum, lowest index on equal distance.
// xlo / xhi hold features 8q..8q+3 and 8q+4..8q+7 of the point, so every lane adds the terms
// in feature order and identical centroids give bit-identical distances whichever lane
// evaluates them.  Rows come from `base` with `stride` floats per row (LDS chunk or global C).
template <int NQ>
__device__ __forceinline__ void eval_group(const floatx4 (&xlo)[NQ], const floatx4 (&xhi)[NQ],
                                           const float *base, int stride, int jfirst, int K, int D,
                                           int g, float &dbest, int &jbest)
{
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int j = jfirst + Mma<float>::row(r, g);
        if (j < K) {
            const float *c = base + (size_t)Mma<float>::row(r, g) * stride;
            float d = 0.f;
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                if (8 * q < D) {
                    const floatx4 cl = *reinterpret_cast<const floatx4 *>(c + 8 * q);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float t = xlo[q][e] - cl[e];
                        d = fmaf(t, t, d);
                    }
                }
                if (8 * q + 4 < D) {
                    const floatx4 ch = *reinterpret_cast<const floatx4 *>(c + 8 * q + 4);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float t = xhi[q][e] - ch[e];
                        d = fmaf(t, t, d);
                    }
                }
            }
            const bool better = d < dbest || (d == dbest && j < jbest);
            dbest = better ? d : dbest;
            jbest = better ? j : jbest;
        }
    }
}

template <int NQ, int PT>
__global__ __launch_bounds__(256) void assign_smalld_kernel(SmallArgs a)
{
    using M = Mma<float>;
    constexpr int SW = 8 * NQ + 4;  // LDS row stride in floats (16 bytes of padding)
    extern __shared__ __align__(16) float lds[];
    float *ldsC = lds;                          // [kch][SW]
    float *ldsH = lds + (size_t)a.kch * SW;     // [kch] -||c||^2/2 in (tile, group, register) order

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int col = lane & 31;
    const int g = lane >> 5;
    const int D = a.D;
    const int tiles_total = (a.K + 31) / 32;
    const int tiles_per_chunk = a.kch / 32;
    const float cmax2 = (float)a.scal[0];
    const float cmax = sqrtf(cmax2);
    int n_refined = 0;

    for (int blk = blockIdx.x; blk < a.nblocks; blk += gridDim.x) {
        const int64_t p0 = ((int64_t)blk * 4 + wave) * (PT * 32);
        floatx4 xf[PT][NQ];
        float xn[PT];
        Top3<float> best[PT];
#pragma unroll
        for (int pt = 0; pt < PT; ++pt) {
            int64_t p = p0 + pt * 32 + col;
            if (p >= a.N) p = a.N - 1;
            const float *xrow = a.X + p * D;
            xn[pt] = 0.f;
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                xf[pt][q] = load_frag<float, true>(xrow, 8 * q + 4 * g, D);
#pragma unroll
                for (int e = 0; e < 4; ++e) xn[pt] = fmaf(xf[pt][q][e], xf[pt][q][e], xn[pt]);
            }
            best[pt].m1 = best[pt].m2 = best[pt].m3 = M::neg_inf();
            best[pt].i1 = best[pt].i2 = 0;
        }

        for (int ch = 0; ch < a.nch; ++ch) {
            if (a.nch > 1 || blk == (int)blockIdx.x) {
                // (re)stage the centroid chunk; with a single chunk it stays resident
                __syncthreads();
                const int jbase = ch * a.kch;
                constexpr int PPR = 2 * NQ;  // 16-byte pieces per row
                for (int idx = tid; idx < a.kch * PPR; idx += 256) {
                    const int rrow = idx / PPR, pc = idx % PPR;
                    const int j = jbase + rrow;
                    floatx4 f = {0.f, 0.f, 0.f, 0.f};
                    if (j < a.K) f = load_frag<float, true>(a.C + (size_t)j * D, 4 * pc, D);
                    *reinterpret_cast<floatx4 *>(ldsC + (size_t)rrow * SW + 4 * pc) = f;
                }
                for (int idx = tid; idx < a.kch; idx += 256) {
                    const int t = idx >> 5, gg = (idx >> 4) & 1, r = idx & 15;
                    ldsH[idx] = -a.hcn[jbase + t * 32 + M::row(r, gg)];
                }
                __syncthreads();
            }
            const int tile0 = ch * tiles_per_chunk;
            const int ntile = min(tiles_per_chunk, tiles_total - tile0);
            for (int t = 0; t < ntile; ++t) {
                floatx4 av[NQ];
#pragma unroll
                for (int q = 0; q < NQ; ++q)
                    av[q] = *reinterpret_cast<const floatx4 *>(ldsC + (size_t)(t * 32 + col) * SW + 8 * q + 4 * g);
                floatx16 cinit;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const floatx4 h = *reinterpret_cast<const floatx4 *>(ldsH + t * 32 + g * 16 + 4 * i);
                    cinit[4 * i + 0] = h[0];
                    cinit[4 * i + 1] = h[1];
                    cinit[4 * i + 2] = h[2];
                    cinit[4 * i + 3] = h[3];
                }
#pragma unroll
                for (int pt = 0; pt < PT; ++pt) {
                    floatx16 acc = cinit;
#pragma unroll
                    for (int q = 0; q < NQ; ++q)
#pragma unroll
                        for (int e = 0; e < 4; ++e) acc = M::mma(av[q][e], xf[pt][q][e], acc);
                    float tm = max3f(acc[0], acc[1], acc[2]);
                    tm = max3f(tm, acc[3], acc[4]);
                    tm = max3f(tm, acc[5], acc[6]);
                    tm = max3f(tm, acc[7], acc[8]);
                    tm = max3f(tm, acc[9], acc[10]);
                    tm = max3f(tm, acc[11], acc[12]);
                    tm = max3f(tm, acc[13], acc[14]);
                    tm = __builtin_fmaxf(tm, acc[15]);
                    best[pt] = top3_insert<float>(best[pt], tm, tile0 + t);
                }
            }
        }

        // ---- exact evaluation of the candidate groups ----
        const bool resident = a.nch == 1;
#pragma unroll
        for (int pt = 0; pt < PT; ++pt) {
            const int64_t p = p0 + pt * 32 + col;
            const bool live = p < a.N;
            floatx4 xlo[NQ], xhi[NQ];
#pragma unroll
            for (int q = 0; q < NQ; ++q)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float mine = xf[pt][q][e];
                    const float other = __shfl_xor(mine, 32, 64);
                    xlo[q][e] = g == 0 ? mine : other;
                    xhi[q][e] = g == 0 ? other : mine;
                }
            const float xnt = xn[pt] + __shfl_xor(xn[pt], 32, 64);
            const float top = fmaxf(best[pt].m1, __shfl_xor(best[pt].m1, 32, 64));
            const float bound = (float)a.band_coef * (sqrtf(xnt) * cmax + 0.5f * cmax2);
            const float thr = top - bound;
            const bool use1 = best[pt].m1 >= thr;
            const bool use2 = best[pt].m2 >= thr;
            const bool over = best[pt].m3 >= thr;
            float dbest = __builtin_huge_valf();
            int jbest = 0x7fffffff;
            if (use1) {
                const int T = best[pt].i1;
                const float *base = resident ? ldsC + (size_t)T * 32 * SW : a.C + (size_t)T * 32 * D;
                eval_group<NQ>(xlo, xhi, base, resident ? SW : D, T * 32, a.K, D, g, dbest, jbest);
            }
            if (use2) {
                const int T = best[pt].i2;
                const float *base = resident ? ldsC + (size_t)T * 32 * SW : a.C + (size_t)T * 32 * D;
                eval_group<NQ>(xlo, xhi, base, resident ? SW : D, T * 32, a.K, D, g, dbest, jbest);
            }
            const float od = __shfl_xor(dbest, 32, 64);
            const int oj = __shfl_xor(jbest, 32, 64);
            if (od < dbest || (od == dbest && oj < jbest)) {
                dbest = od;
                jbest = oj;
            }
            const bool over_any = over || (__shfl_xor((int)over, 32, 64) != 0);
            const bool two_any = use2 || (__shfl_xor((int)use2, 32, 64) != 0);
            if (live && g == 0) {
                a.labels[p] = jbest == 0x7fffffff ? 0 : jbest;
                if (a.mindist) a.mindist[p] = dbest;
                if (over_any) {
                    const int pos = atomicAdd(a.wl_count, 1);
                    a.wl[pos] = (int32_t)p;
                } else if (two_any) {
                    n_refined += 1;
                }
            }
        }
    }
    if (a.stats) {
        int n = n_refined;
#pragma unroll
        for (int mask = 1; mask < 64; mask <<= 1) n += __shfl_xor(n, mask, 64);
        if (lane == 0 && n) atomicAdd((unsigned long long *)&a.stats->refined, (unsigned long long)n);
    }
}

bool smalld_supported(ftk_dtype dtype, int D, int K)
{
    (void)K;
    return dtype == FTK_F32 && D <= 32 && D % 4 == 0;
}

static int smalld_pt(int D8) { return D8 <= 16 ? 2 : 2; }

void plan_smalld(int64_t N, int D, int K, ftk_ft_mode ft, AssignPlan &p)
{
    (void)ft;
    p.variant = VAR_SMALLD;
    p.TM = 32;
    p.TN = 32;
    p.D8 = (int)ceil_div(D, 8) * 8;
    p.PT = smalld_pt(p.D8);
    p.KT = 1;
    p.waves = 4;
    const int SW = p.D8 + 4;
    // chunk: as many centroids as fit 64 KB of LDS, all of them if possible
    int kch = (64 * 1024) / (SW * 4 + 4) / 32 * 32;
    const int Kr = (int)ceil_div(K, 32) * 32;
    if (kch > Kr) kch = Kr;
    p.kch = kch;
    p.KC = kch;
    p.nkc = (int)ceil_div(K, kch);
    p.DQ = p.D8 / 8;
    p.points_per_wg = 4 * p.PT * 32;
    p.workgroups = ceil_div(N, p.points_per_wg);
    p.lds_bytes = (size_t)kch * (SW * 4 + 4);
    int resident_wgs = (int)(160 * 1024 / (p.lds_bytes + 512));
    if (resident_wgs > 4) resident_wgs = 4;
    if (resident_wgs < 1) resident_wgs = 1;
    const int64_t cap = 256LL * resident_wgs;
    p.grid = (int)(p.workgroups < cap ? p.workgroups : cap);
    p.tiles_per_wave = (int)(ceil_div(K, 32) * p.PT * ceil_div(p.workgroups, p.grid));
    p.regs_per_tile = 16;
    p.hcn_pad_inf = true;
}

template <int NQ, int PT>
static void launch_smalld_t(const SmallArgs &a, const AssignPlan &p, hipStream_t st)
{
    hipLaunchKernelGGL((assign_smalld_kernel<NQ, PT>), dim3(p.grid), dim3(256), p.lds_bytes, st, a);
}

ftk_status launch_assign_smalld(const AssignCall &c, const AssignPlan &p, const Workspace &w, hipStream_t st)
{
    if ((uintptr_t)c.X % 16 || (uintptr_t)c.C % 16) {
        set_error("small-D variant needs 16-byte aligned X and C");
        return FTK_EALIGN;
    }
    SmallArgs a;
    a.X = (const float *)c.X;
    a.C = (const float *)c.C;
    a.hcn = (const float *)w.hcn;
    a.scal = w.scal;
    a.N = c.N;
    a.D = c.D;
    a.K = c.K;
    a.kch = p.kch;
    a.nch = p.nkc;
    a.nblocks = (int)p.workgroups;
    a.labels = c.labels;
    a.mindist = (float *)c.mindist;
    a.wl = w.wl;
    a.wl_count = w.wl_count;
    a.stats = c.stats;
    a.band_coef = 4.0 * (c.D + 4) * Mma<float>::kEps;
    switch (p.D8 / 8) {
    case 1: launch_smalld_t<1, 2>(a, p, st); break;
    case 2: launch_smalld_t<2, 2>(a, p, st); break;
    case 3: launch_smalld_t<3, 2>(a, p, st); break;
    default: launch_smalld_t<4, 2>(a, p, st); break;
    }
    FTK_TRY_HIP(hipGetLastError());
    return FTK_OK;
}

}  // namespace ftk
