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
#include <cstdlib>
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
    int dbg;
};

__device__ __forceinline__ float max3f(float a, float b, float c) { return __builtin_fmaxf(__builtin_fmaxf(a, b), c); }

// Exact (direct-difference, fp32) distances of one point to 8 centroids of one lane group's
// share of a tile: registers r0..r0+7 of group gw in the tile whose rows start at `base`
// (`stride` floats per row, LDS chunk or global C).  xlo / xhi hold features 8q..8q+3 and
// 8q+4..8q+7 of the point, so terms are always added in feature order and identical centroids
// give bit-identical distances whichever lane evaluates them.  Keeps the running (distance,
// index) minimum, lowest index on equal distance.
template <int NQ, bool PADDED>
__device__ __forceinline__ void eval_rows(const floatx4 (&xlo)[NQ], const floatx4 (&xhi)[NQ],
                                          const float *base, int stride, int jfirst, int K, int D,
                                          int gw, int r0, float &dbest, int &jbest)
{
    // PADDED: rows are zero-padded to 8*NQ features (LDS copy), no bounds checks needed; the
    // point fragments are zero beyond D as well.
    float d[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        // register r = r0 + i of group gw holds tile row 8*(r/4) + 4*gw + r%4; r0 is 0 or 8
        const int row = 8 * (i >> 2) + (i & 3) + 2 * r0 + 4 * gw;
        const float *c = base + row * stride;
        d[i] = 0.f;
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            floatx4 cl = {0.f, 0.f, 0.f, 0.f}, ch = {0.f, 0.f, 0.f, 0.f};
            if (PADDED || (8 * q < D && jfirst + row < K)) cl = *reinterpret_cast<const floatx4 *>(c + 8 * q);
            if (PADDED || (8 * q + 4 < D && jfirst + row < K)) ch = *reinterpret_cast<const floatx4 *>(c + 8 * q + 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float t = xlo[q][e] - cl[e];
                d[i] = fmaf(t, t, d[i]);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float t = xhi[q][e] - ch[e];
                d[i] = fmaf(t, t, d[i]);
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int j = jfirst + 8 * (i >> 2) + (i & 3) + 2 * r0 + 4 * gw;
        const float db = dbest;
        const int jb = jbest;
        const bool better = (j < K) & ((d[i] < db) | ((d[i] == db) & (j < jb)));
        dbest = better ? d[i] : db;
        jbest = better ? j : jb;
    }
}

constexpr int SMALLD_WAVES = 8;  // waves per workgroup sharing one staged centroid chunk
constexpr int SMALLD_THREADS = SMALLD_WAVES * 64;

// Best tile maximum, the tile it came from, and the runner-up tile maximum of one lane.
struct TileBest {
    float m1, m2;
    int t1;
};

template <int NQ, int PT>
__global__ __launch_bounds__(SMALLD_THREADS) void assign_smalld_kernel(SmallArgs a)
{
    using M = Mma<float>;
    constexpr int SW = 8 * NQ + 4;      // LDS row stride in floats (16 bytes of padding)
    constexpr int TS = 32 * SW + 4;     // LDS tile stride: 16 more bytes so that lanes reading rows
                                        // of different tiles (exact re-evaluation) spread over banks
    extern __shared__ __align__(16) float lds[];
    const int tiles_per_chunk = a.kch / 32;
    float *ldsC = lds;                                  // [tiles_per_chunk][TS]
    float *ldsH = lds + (size_t)tiles_per_chunk * TS;   // [kch] -||c||^2/2 in (tile, group, register) order

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int col = lane & 31;
    const int g = lane >> 5;
    const int D = a.D;
    const int tiles_total = (a.K + 31) / 32;
    const float cmax2 = (float)a.scal[0];
    const float cmax = sqrtf(cmax2);
    int n_refined = 0;

    // operand fetch of one centroid tile: A fragments and the accumulator start values
    auto load_tile = [&](int t, floatx4 (&av)[NQ], floatx16 &ci) {
        const float *rowp = ldsC + (size_t)t * TS + col * SW + 4 * g;
#pragma unroll
        for (int q = 0; q < NQ; ++q) av[q] = *reinterpret_cast<const floatx4 *>(rowp + 8 * q);
        const float *hp = ldsH + t * 32 + g * 16;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const floatx4 h = *reinterpret_cast<const floatx4 *>(hp + 4 * i);
            ci[4 * i + 0] = h[0];
            ci[4 * i + 1] = h[1];
            ci[4 * i + 2] = h[2];
            ci[4 * i + 3] = h[3];
        }
    };

    // Blocks of SMALLD_WAVES units (PT*32 points per wave) are handed out dynamically from an
    // atomic counter so that nothing idles while a queue remains.  The waves of a workgroup
    // deliberately stay in step (one barrier per block): on this hardware fp32 matrix and
    // vector instructions share the issue path, and waves that drift into different phases
    // (one multiplying, one reducing) interleave them finely, which measurably costs throughput.
    __shared__ int sh_next;
    const bool resident = a.nch == 1;
    auto stage_chunk = [&](int ch) {
        const int jbase = ch * a.kch;
        constexpr int PPR = 2 * NQ;  // 16-byte pieces per row
        for (int idx = tid; idx < a.kch * PPR; idx += SMALLD_THREADS) {
            const int rrow = idx / PPR, pc = idx % PPR;
            const int j = jbase + rrow;
            floatx4 f = {0.f, 0.f, 0.f, 0.f};
            if (j < a.K) f = load_frag<float, true>(a.C + (size_t)j * D, 4 * pc, D);
            *reinterpret_cast<floatx4 *>(ldsC + (size_t)(rrow >> 5) * TS + (rrow & 31) * SW + 4 * pc) = f;
        }
        for (int idx = tid; idx < a.kch; idx += SMALLD_THREADS) {
            const int t = idx >> 5, gg = (idx >> 4) & 1, r = idx & 15;
            ldsH[idx] = -a.hcn[jbase + t * 32 + M::row(r, gg)];
        }
    };
    if (resident) {
        stage_chunk(0);
        __syncthreads();
    }
    int blk = blockIdx.x;
    while (blk < a.nblocks) {
        const int64_t p0 = ((int64_t)blk * SMALLD_WAVES + wave) * (PT * 32);
        floatx4 xf[PT][NQ];
        float xn[PT];
        TileBest best[PT];
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
            best[pt].m1 = best[pt].m2 = M::neg_inf();
            best[pt].t1 = 0;
        }

        // one output tile: contraction, tile maximum per lane, running best tile
        auto compute_tile = [&](const floatx4 (&av)[NQ], const floatx16 &ci, int tile) {
#pragma unroll
            for (int pt = 0; pt < PT; ++pt) {
                floatx16 acc = ci;
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
                const float m1 = best[pt].m1, m2 = best[pt].m2;
                const int t1 = best[pt].t1;
                const bool c = tm > m1;
                best[pt].m2 = __builtin_amdgcn_fmed3f(m1, m2, tm);
                best[pt].t1 = c ? tile : t1;
                best[pt].m1 = __builtin_fmaxf(m1, tm);
            }
        };

        for (int ch = 0; ch < a.nch; ++ch) {
            if (!resident) {
                __syncthreads();  // every wave is done with the previous chunk
                stage_chunk(ch);
                __syncthreads();
            }
            const int tile0 = ch * tiles_per_chunk;
            const int ntile = min(tiles_per_chunk, tiles_total - tile0);
            // two operand register sets: the fetch of the next tile is in flight while the
            // current one is multiplied
            floatx4 avA[NQ], avB[NQ];
            floatx16 ciA, ciB;
            load_tile(0, avA, ciA);
            for (int t = 0; t < ntile; t += 2) {
                load_tile(min(t + 1, ntile - 1), avB, ciB);
                compute_tile(avA, ciA, tile0 + t);
                load_tile(min(t + 2, ntile - 1), avA, ciA);
                if (t + 1 < ntile) compute_tile(avB, ciB, tile0 + t + 1);
            }
        }

        // ---- exact evaluation of the winning group; the two lanes of a point share its rows ----
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
            const float bound = (float)a.band_coef * (sqrtf(xnt) * cmax + 0.5f * cmax2);
            const float om1 = __shfl_xor(best[pt].m1, 32, 64), om2 = __shfl_xor(best[pt].m2, 32, 64);
            const int ot1 = __shfl_xor(best[pt].t1, 32, 64);
            const bool mine_wins = best[pt].m1 > om1 || (best[pt].m1 == om1 && g == 0);
            const float thr = fmaxf(best[pt].m1, om1) - bound;
            // first round: the group holding the best tile maximum (gw = its lane group)
            const int gw = mine_wins ? g : 1 - g;
            const int Tw = mine_wins ? best[pt].t1 : ot1;
            // second round (rare): the other group's best tile is inside the bound as well
            const bool second = fminf(best[pt].m1, om1) >= thr;
            const int Ts = mine_wins ? ot1 : best[pt].t1;
            // a third candidate tile anywhere: left to the refine kernel
            const bool over = fmaxf(best[pt].m2, om2) >= thr;
            float dbest = __builtin_huge_valf();
            int jbest = 0x7fffffff;
            if (resident) {
                eval_rows<NQ, true>(xlo, xhi, ldsC + Tw * TS, SW, Tw * 32, a.K, D, gw, 8 * g, dbest, jbest);
                if (__any(second)) {
                    float d2 = dbest;
                    int j2 = jbest;
                    eval_rows<NQ, true>(xlo, xhi, ldsC + Ts * TS, SW, Ts * 32, a.K, D, 1 - gw, 8 * g, d2, j2);
                    dbest = second ? d2 : dbest;
                    jbest = second ? j2 : jbest;
                }
            } else {
                eval_rows<NQ, false>(xlo, xhi, a.C + (size_t)Tw * 32 * D, D, Tw * 32, a.K, D, gw, 8 * g, dbest, jbest);
                if (__any(second)) {
                    float d2 = dbest;
                    int j2 = jbest;
                    eval_rows<NQ, false>(xlo, xhi, a.C + (size_t)Ts * 32 * D, D, Ts * 32, a.K, D, 1 - gw, 8 * g, d2, j2);
                    dbest = second ? d2 : dbest;
                    jbest = second ? j2 : jbest;
                }
            }
            const float od = __shfl_xor(dbest, 32, 64);
            const int oj = __shfl_xor(jbest, 32, 64);
            const bool take = (od < dbest) | ((od == dbest) & (oj < jbest));
            dbest = take ? od : dbest;
            jbest = take ? oj : jbest;
            if (live && g == 0) {
                a.labels[p] = jbest == 0x7fffffff ? 0 : jbest;
                if (a.mindist) a.mindist[p] = dbest;
                if (!(thr == thr) || over) {   // NaN scores or a third candidate tile
                    const int pos = atomicAdd(a.wl_count, 1);
                    a.wl[pos] = (int32_t)p;
                }
            }
        }
        __syncthreads();
        if (tid == 0) sh_next = (int)gridDim.x + atomicAdd(a.wl_count + 1, 1);
        __syncthreads();
        blk = sh_next;
    }
    (void)n_refined;
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
    p.waves = SMALLD_WAVES;
    const int SW = p.D8 + 4;
    // chunk: as many centroids as fit 64 KB of LDS, all of them if possible
    int kch = (64 * 1024) / (SW * 4 + 4 + 1) / 32 * 32;
    const int Kr = (int)ceil_div(K, 32) * 32;
    if (kch > Kr) kch = Kr;
    p.kch = kch;
    p.KC = kch;
    p.nkc = (int)ceil_div(K, kch);
    p.DQ = p.D8 / 8;
    p.points_per_wg = SMALLD_WAVES * p.PT * 32;
    p.workgroups = ceil_div(N, p.points_per_wg);
    p.lds_bytes = (size_t)(kch / 32) * (32 * SW + 4) * 4 + (size_t)kch * 4;
    int resident_wgs = (int)(160 * 1024 / (p.lds_bytes + 2048));
    if (resident_wgs > 2) resident_wgs = 2;
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
    hipLaunchKernelGGL((assign_smalld_kernel<NQ, PT>), dim3(p.grid), dim3(SMALLD_THREADS), p.lds_bytes, st, a);
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
    a.dbg = getenv("FTK_DBG") ? atoi(getenv("FTK_DBG")) : 0;
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
