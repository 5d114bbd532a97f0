// Fast assignment for fp32 data with D <= 32: the contraction runs on the bf16 matrix
// instructions (16 times the fp32 rate on this hardware), with both operands split into three
// bf16 pieces so that almost nothing of the fp32 product is lost.  It plays the part the paper
// gives to its TF32 tensor-core path (Section 3.1.5: reduced-precision inputs, fp32
// accumulation) - gfx950 has no TF32 format - but keeps the exactness of the fp32 path: the
// rounding bound below is certified, and points whose best scores fall inside it are settled by
// exact re-evaluation exactly as in the fp32 kernel, so the labels meet the same tie tolerance.
//
// Split: x = x0 + x1 + x2 with x0 = bf16(x), x1 = bf16(x - x0), x2 = bf16(x - x0 - x1); the
// three pieces carry 8 significant bits each, so the sum is x itself.  Of the nine piece
// products the six largest are kept,
//     x.c ~ x0c0 + x0c1 + x1c0 + x0c2 + x1c1 + x2c0        (dropped: at most 2^-24 |x_d c_d| each feature)
// and laid along the contraction index of the 32x32x16 instruction: lane group 0 supplies
// k = 0..7, lane group 1 k = 8..15, so one instruction takes two (piece, piece) pairs of one
// block of 8 features:
//     instruction 1:  A = (c0 | c1)  B = (x0 | x0)      instruction 2:  A = (c0 | c1)  B = (x1 | x1)
//     instruction 3:  A = (c2 | c0)  B = (x0 | x2)
// i.e. two A fragments per block from LDS (the centroid pieces are prepared once per call by
// split_centroids_kernel, already in LDS image order) and three B fragments per block held in
// registers for the whole sweep.  Output layout, start values -||c||^2/2, tile maximum, best
// tile and the exact settlement are those of the fp32 small-D kernel.
//
// Rounding bound (measured on the device, not documented): the instruction aligns its 17 addends
// (16 products, which are exact, and the accumulator) to the largest exponent keeping three
// guard bits and truncates the rest, then rounds the sum to fp32.  Each addend loses less than
// 2^-26 of the largest, the final rounding at most 2^-23 of the result: |error| <= 6.25 u M per
// instruction with u = 2^-24 and M = |accumulator| + sum |products|; random operands show 3.3 u M.
// The launcher budgets 7 u per instruction plus 2 u for the dropped products.
#include <cmath>

#include "ftk_internal.h"
#include "ftk_mma.h"
#include "ftk_smalld.h"

namespace ftk {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct FastArgs {
    const float *X;
    const float *C;
    const float *hcn;     // half squared norms of the K centroids
    const double *scal;   // scal[0] = max_j ||c_j||^2
    const uint4 *csplit;  // [tiles_total][32][row units] centroid pieces, 16-byte units
    int64_t N;
    int D, K;
    int tpc;          // tiles staged in LDS at a time
    int nch;          // chunks
    int tiles_total;  // ceil(K / 32)
    int nblocks;      // point blocks (waves*PT*32 points each)
    int nunits;       // wave units (PT*32 points each)
    int32_t *labels;
    float *mindist;
    int32_t *wl;
    int32_t *wl_count;
    double band_coef;
};

// 16-byte units per centroid row in the LDS image: 3 pieces of NQ blocks, padded to an odd count
// so that the 32 rows of a tile spread over the banks
static constexpr int fast_row_units(int nq) { return (3 * nq + 1) % 2 ? 3 * nq + 1 : 3 * nq + 2; }
// One workgroup per CU: 16 waves (4 per SIMD, 128 registers) for D <= 8, else 8 waves (2 per SIMD,
// 256 registers for the point fragments); two point tiles per wave.  Measured alternatives for
// D = 8 (8 waves, four point tiles per wave) came out within 5 %.
static constexpr int fast_waves(int nq) { return nq == 1 ? 16 : 8; }
static constexpr int fast_waves_per_simd(int nq) { return nq == 1 ? 4 : 2; }
static constexpr int fast_pt(int nq) { (void)nq; return 2; }

__device__ __forceinline__ void split3(float x, __bf16 &p0, __bf16 &p1, __bf16 &p2)
{
    p0 = (__bf16)x;
    float r = x - (float)p0;  // exact: p0 agrees with x in its leading bits
    p1 = (__bf16)r;
    r -= (float)p1;           // exact, at most 8 significant bits are left
    p2 = (__bf16)r;
}

// Centroid pieces in LDS image order.  One thread per (row of the padded K, block of 8 features).
template <int NQ>
__global__ __launch_bounds__(256) void split_centroids_kernel(const float *C, int D, int K, int rows, uint4 *img)
{
    constexpr int SU = fast_row_units(NQ);
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= rows * NQ) return;
    const int row = t / NQ, b = t % NQ;
    bf16x8 p0, p1, p2;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int d = 8 * b + e;
        const float v = (row < K && d < D) ? C[(size_t)row * D + d] : 0.f;
        __bf16 q0, q1, q2;
        split3(v, q0, q1, q2);
        p0[e] = q0;
        p1[e] = q1;
        p2[e] = q2;
    }
    uint4 *dst = img + (size_t)row * SU;  // tiles are 32 consecutive rows
    dst[b] = __builtin_bit_cast(uint4, p0);
    dst[NQ + b] = __builtin_bit_cast(uint4, p1);
    dst[2 * NQ + b] = __builtin_bit_cast(uint4, p2);
}

template <int NQ, int PT>
__global__ __launch_bounds__(fast_waves(NQ) * 64, fast_waves_per_simd(NQ)) void assign_fast_kernel(FastArgs a)
{
    constexpr int WAVES = fast_waves(NQ);
    constexpr int THREADS = WAVES * 64;
    constexpr int SU = fast_row_units(NQ);
    constexpr int TU = 32 * SU;  // units per tile
    using M = Mma<float>;
    extern __shared__ __align__(16) uint4 lds4[];
    uint4 *ldsC = lds4;                                           // [tpc][TU]
    float *ldsH = reinterpret_cast<float *>(lds4 + (size_t)a.tpc * TU);  // [tpc*32] start values, (tile, group, register) order
    __shared__ int sh_next;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int col = lane & 31;
    const int g = lane >> 5;
    const int D = a.D;
    const float cmax2 = (float)a.scal[0];
    const float cmax = sqrtf(cmax2);
    const bool resident = a.nch == 1;

    // A fragments of one tile: (c0 | c1) and (c2 | c0) per block, plus the accumulator start values
    // (per-lane bases, so that every read of a tile is one base plus a constant offset)
    const uint4 *base0 = ldsC + col * SU + (g ? NQ : 0);
    const uint4 *base1 = ldsC + col * SU + (g ? 0 : 2 * NQ);
    auto load_tile = [&](int t, uint4 (&t0)[NQ], uint4 (&t1)[NQ], floatx16 &ci) {
        const uint4 *p0 = base0 + t * TU;
        const uint4 *p1 = base1 + t * TU;
#pragma unroll
        for (int b = 0; b < NQ; ++b) {
            t0[b] = p0[b];
            t1[b] = p1[b];
        }
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

    auto stage_chunk = [&](int ch) {
        const int tile0 = ch * a.tpc;
        const int ntile = min(a.tpc, a.tiles_total - tile0);
        const uint4 *src = a.csplit + (size_t)tile0 * TU;
        for (int idx = tid; idx < ntile * TU; idx += THREADS) ldsC[idx] = src[idx];
        for (int idx = tid; idx < ntile * 32; idx += THREADS) {
            const int tl = idx >> 5, gg = (idx >> 4) & 1, r = idx & 15;
            const int j = 32 * (tile0 + tl) + M::row(r, gg);
            ldsH[idx] = j < a.K ? -a.hcn[j] : M::neg_inf();
        }
    };
    if (resident) {
        stage_chunk(0);
        __syncthreads();
    }

    // all the work on one unit of PT*32 points
    auto process = [&](int unit) {
        const int64_t p0 = (int64_t)unit * (PT * 32);
        uint4 s0[PT][NQ], s1[PT][NQ], s2[PT][NQ];  // B fragments: (x0 | x0), (x1 | x1), (x0 | x2)
        float xn[PT];
        TileBest best[PT];
#pragma unroll
        for (int pt = 0; pt < PT; ++pt) {
            int64_t p = p0 + pt * 32 + col;
            if (p >= a.N) p = a.N - 1;
            const float *xrow = a.X + p * D;
            float s = 0.f;
#pragma unroll
            for (int b = 0; b < NQ; ++b) {
                const floatx4 lo = load_frag<float, true>(xrow, 8 * b, D);
                const floatx4 hi = load_frag<float, true>(xrow, 8 * b + 4, D);
                bf16x8 q0, q1, q2;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float v = e < 4 ? lo[e] : hi[e - 4];
                    s = fmaf(v, v, s);
                    __bf16 u0, u1, u2;
                    split3(v, u0, u1, u2);
                    q0[e] = u0;
                    q1[e] = u1;
                    q2[e] = u2;
                }
                s0[pt][b] = __builtin_bit_cast(uint4, q0);
                s1[pt][b] = __builtin_bit_cast(uint4, q1);
                const uint4 w2 = __builtin_bit_cast(uint4, q2);
                s2[pt][b].x = g ? w2.x : s0[pt][b].x;
                s2[pt][b].y = g ? w2.y : s0[pt][b].y;
                s2[pt][b].z = g ? w2.z : s0[pt][b].z;
                s2[pt][b].w = g ? w2.w : s0[pt][b].w;
            }
            xn[pt] = s;
            best[pt].m1 = best[pt].m2 = M::neg_inf();
            best[pt].t1 = 0;
        }

        auto compute_tile = [&](const uint4 (&t0)[NQ], const uint4 (&t1)[NQ], const floatx16 &ci, int T) {
            floatx16 accs[PT];
#pragma unroll
            for (int pt = 0; pt < PT; ++pt) accs[pt] = ci;
            // smallest products first; the PT accumulator chains are independent and interleave
#pragma unroll
            for (int b = 0; b < NQ; ++b)
#pragma unroll
                for (int pt = 0; pt < PT; ++pt)
                    accs[pt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, t1[b]),
                                                                       __builtin_bit_cast(bf16x8, s2[pt][b]), accs[pt], 0, 0, 0);
#pragma unroll
            for (int b = 0; b < NQ; ++b)
#pragma unroll
                for (int pt = 0; pt < PT; ++pt)
                    accs[pt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, t0[b]),
                                                                       __builtin_bit_cast(bf16x8, s1[pt][b]), accs[pt], 0, 0, 0);
#pragma unroll
            for (int b = 0; b < NQ; ++b)
#pragma unroll
                for (int pt = 0; pt < PT; ++pt)
                    accs[pt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, t0[b]),
                                                                       __builtin_bit_cast(bf16x8, s0[pt][b]), accs[pt], 0, 0, 0);
#pragma unroll
            for (int pt = 0; pt < PT; ++pt) {
                const floatx16 acc = accs[pt];
                float tm = max2f(acc[0], acc[1]);
#pragma unroll
                for (int r = 2; r < 16; r += 2) tm = max3f(tm, acc[r], acc[r + 1]);
                const float m1 = best[pt].m1, m2 = best[pt].m2;
                const int t1b = best[pt].t1;
                const bool c = tm > m1;
                best[pt].m2 = __builtin_amdgcn_fmed3f(m1, m2, tm);
                best[pt].t1 = c ? T : t1b;
                best[pt].m1 = max2f(m1, tm);
            }
        };

        for (int ch = 0; ch < a.nch; ++ch) {
            if (!resident) {
                __syncthreads();  // every wave is done with the previous chunk
                stage_chunk(ch);
                __syncthreads();
            }
            const int tile0 = ch * a.tpc;
            const int ntile = min(a.tpc, a.tiles_total - tile0);
            if constexpr (NQ <= 2) {
                // two operand register sets: the fetch of the next tile is in flight during the current one
                uint4 t0A[NQ], t1A[NQ], t0B[NQ], t1B[NQ];
                floatx16 ciA, ciB;
                load_tile(0, t0A, t1A, ciA);
                for (int t = 0; t < ntile; t += 2) {
                    load_tile(min(t + 1, ntile - 1), t0B, t1B, ciB);
                    compute_tile(t0A, t1A, ciA, tile0 + t);
                    load_tile(min(t + 2, ntile - 1), t0A, t1A, ciA);
                    if (t + 1 < ntile) compute_tile(t0B, t1B, ciB, tile0 + t + 1);
                }
            } else {
                // wide rows: one set (the registers are needed for the point fragments); the other
                // wave of the SIMD covers the fetch
                uint4 t0A[NQ], t1A[NQ];
                floatx16 ciA;
                for (int t = 0; t < ntile; ++t) {
                    load_tile(t, t0A, t1A, ciA);
                    compute_tile(t0A, t1A, ciA, tile0 + t);
                }
            }
        }

        // ---- exact evaluation of the winning group; the two lanes of a point share its rows ----
#pragma unroll
        for (int pt = 0; pt < PT; ++pt) {
            const int64_t p = p0 + pt * 32 + col;
            const bool live = p < a.N;
            const float *xrow = a.X + (live ? p : a.N - 1) * D;
            floatx4 xlo[NQ], xhi[NQ];
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                xlo[q] = load_frag<float, true>(xrow, 8 * q, D);
                xhi[q] = load_frag<float, true>(xrow, 8 * q + 4, D);
            }
            const float bound = (float)a.band_coef * (sqrtf(xn[pt]) * cmax + 0.5f * cmax2);
            const float om1 = __shfl_xor(best[pt].m1, 32, 64), om2 = __shfl_xor(best[pt].m2, 32, 64);
            const int ot1 = __shfl_xor(best[pt].t1, 32, 64);
            const bool mine_wins = best[pt].m1 > om1 || (best[pt].m1 == om1 && g == 0);
            const float thr = fmaxf(best[pt].m1, om1) - bound;
            const int gw = mine_wins ? g : 1 - g;
            const int Tw = mine_wins ? best[pt].t1 : ot1;
            const bool second = fminf(best[pt].m1, om1) >= thr;
            const int Ts = mine_wins ? ot1 : best[pt].t1;
            const bool over = fmaxf(best[pt].m2, om2) >= thr;
            float dbest = __builtin_huge_valf();
            int jbest = 0x7fffffff;
            eval_rows<NQ, false, false>(xlo, xhi, a.C, D, Tw, a.K, D, gw, 8 * g, dbest, jbest);
            if (__any(second)) {
                float d2 = dbest;
                int j2 = jbest;
                eval_rows<NQ, false, false>(xlo, xhi, a.C, D, Ts, a.K, D, 1 - gw, 8 * g, d2, j2);
                dbest = second ? d2 : dbest;
                jbest = second ? j2 : jbest;
            }
            const float od = __shfl_xor(dbest, 32, 64);
            const int oj = __shfl_xor(jbest, 32, 64);
            const bool take = (od < dbest) | ((od == dbest) & (oj < jbest));
            dbest = take ? od : dbest;
            jbest = take ? oj : jbest;
            if (live && g == 0) {
                a.labels[p] = jbest == 0x7fffffff ? 0 : jbest;
                if (a.mindist) a.mindist[p] = dbest;
            }
            // NaN scores or a third candidate: exact recomputation
            worklist_push(live && g == 0 && (!(thr == thr) || over), (int32_t)p, a.wl, a.wl_count);
        }
    };

    if (resident) {
        // Every centroid tile stays in LDS: the waves need no common step.  Each takes every
        // (grid * WAVES)-th unit - equal work per unit, so a fixed split balances, and a counter
        // drawn by every wave would cost one device-wide atomic per 64 points - and one wave's
        // exact settlement (a chain of memory latencies) runs under the matrix work of the others.
        for (int unit = (int)blockIdx.x * WAVES + wave; unit < a.nunits; unit += (int)gridDim.x * WAVES) process(unit);
    } else {
        // chunks are staged by the whole workgroup: its waves walk the point blocks together
        int blk = blockIdx.x;
        while (blk < a.nblocks) {
            process(blk * WAVES + wave);
            __syncthreads();
            if (tid == 0) sh_next = (int)gridDim.x + atomicAdd(a.wl_count + 1, 1);
            __syncthreads();
            blk = sh_next;
        }
    }
}

bool fast_supported(ftk_dtype dtype, int D)
{
    return dtype == FTK_F32 && D <= 32 && D % 4 == 0;
}

size_t fast_split_bytes(ftk_dtype dtype, int D, int K)
{
    if (!fast_supported(dtype, D)) return 0;
    const int nq = (int)ceil_div(D, 8);
    return (size_t)ceil_div(K, 32) * 32 * fast_row_units(nq) * sizeof(uint4);
}

// The prologue (norms, their maximum, per-call state) is shared with the fp32 path; it only needs
// the extent to which the half-norm vector is padded.
void plan_fast_prologue(int D, int K, AssignPlan &p)
{
    p.variant = VAR_SMALLD;
    p.D8 = (int)ceil_div(D, 8) * 8;
    p.KC = 32;
    p.nkc = (int)ceil_div(K, 32);
    p.hcn_pad_inf = true;
}

template <int NQ>
static void launch_fast_t(FastArgs a, int64_t N, hipStream_t st)
{
    constexpr int PT = fast_pt(NQ);
    constexpr int SU = fast_row_units(NQ);
    const int rows = a.tiles_total * 32;
    hipLaunchKernelGGL((split_centroids_kernel<NQ>), dim3((unsigned)ceil_div((int64_t)rows * NQ, 256)), dim3(256), 0, st,
                       a.C, a.D, a.K, rows, const_cast<uint4 *>(a.csplit));
    const int tile_bytes = 32 * SU * 16 + 32 * 4;
    // one workgroup per CU; all tiles resident if they fit, else equal chunks
    int tpc = (144 * 1024) / tile_bytes;
    if (tpc > a.tiles_total) tpc = a.tiles_total;
    tpc = (int)ceil_div(a.tiles_total, ceil_div(a.tiles_total, tpc));
    a.tpc = tpc;
    a.nch = (int)ceil_div(a.tiles_total, tpc);
    const int points_per_wg = fast_waves(NQ) * PT * 32;
    a.nblocks = (int)ceil_div(N, points_per_wg);
    a.nunits = (int)ceil_div(N, PT * 32);
    const int grid = a.nblocks < 256 ? a.nblocks : 256;
    hipLaunchKernelGGL((assign_fast_kernel<NQ, PT>), dim3(grid), dim3(fast_waves(NQ) * 64), (size_t)tpc * tile_bytes, st, a);
}

ftk_status launch_assign_fast(const AssignCall &c, const Workspace &w, hipStream_t st)
{
    if ((uintptr_t)c.X % 16 || (uintptr_t)c.C % 16) {
        set_error("the fast variant needs 16-byte aligned X and C");
        return FTK_EALIGN;
    }
    FastArgs a;
    a.X = (const float *)c.X;
    a.C = (const float *)c.C;
    a.hcn = (const float *)w.hcn;
    a.scal = w.scal;
    a.csplit = (const uint4 *)w.csplit;
    a.N = c.N;
    a.D = c.D;
    a.K = c.K;
    a.tiles_total = (int)ceil_div(c.K, 32);
    a.labels = c.labels;
    a.mindist = (float *)c.mindist;
    a.wl = w.wl;
    a.wl_count = w.wl_count;
    const int nq = (int)ceil_div(c.D, 8);
    // two scores, each 3*nq instructions at 7 u of its magnitude, plus 2 u for the dropped
    // products and 2 u for the fp32 evaluation of the magnitude itself
    a.band_coef = 2.0 * (21.0 * nq + 4.0) * Mma<float>::kEps;
    switch (nq) {
    case 1: launch_fast_t<1>(a, c.N, st); break;
    case 2: launch_fast_t<2>(a, c.N, st); break;
    case 3: launch_fast_t<3>(a, c.N, st); break;
    default: launch_fast_t<4>(a, c.N, st); break;
    }
    FTK_TRY_HIP(hipGetLastError());
    return FTK_OK;
}

}  // namespace ftk
