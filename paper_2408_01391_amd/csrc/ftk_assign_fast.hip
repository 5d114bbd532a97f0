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
//
// Fault tolerance (Sections 2.3, 4; the paper protects its tensor-core variant the same way as the
// fp32 one): with FT on, tiles, checksum rows, verification, location and correction are those of
// the fp32 small-D kernel - 30 centroids per tile, register 15 of each lane group carries
// x.(sum of the group's 15 centroids) - sum ||c||^2/2.  The checksum rows are split into bf16
// pieces like any centroid row, so the carried checksum goes through the same instructions as
// the scores it must equal, and the residual's rounding noise is no larger than on the fp32 path
// (same detection threshold).
#include <cmath>
#include <type_traits>

#include "ftk_fast.h"
#include "ftk_internal.h"
#include "ftk_mma.h"
#include "ftk_smalld.h"

namespace ftk {

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

// Centroid pieces in LDS image order.  One thread per (row of the padded tiles, block of 8
// features).  Without checksums row 32T + i holds centroid 32T + i; with them a tile holds 30
// centroids in the rows their accumulator registers read (register r of lane group g sits in row
// 8(r/4) + 4g + r%4) and the two rows of register 15 hold the groups' checksum rows.
template <int NQ, bool FT>
__global__ __launch_bounds__(256) void split_centroids_kernel(const float *C, const float *chk_v1, int D, int K,
                                                              int tiles_total, uint4 *img)
{
    constexpr int SU = fast_row_units(NQ);
    constexpr int D8 = 8 * NQ;
    const int rows = tiles_total * 32;
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= rows * NQ) return;
    const int row = t / NQ, b = t % NQ;
    const float *src = nullptr;
    int width = D;
    if constexpr (FT) {
        const int T = row >> 5, lr = row & 31;
        const int gg = (lr >> 2) & 1, r = (lr >> 3) * 4 + (lr & 3);
        if (r < 15) {
            const int j = 30 * T + 15 * gg + r;
            if (j < K) src = C + (size_t)j * D;
        } else {
            src = chk_v1 + (size_t)(T * 2 + gg) * D8;
            width = D8;
        }
    } else {
        if (row < K) src = C + (size_t)row * D;
    }
    bf16x8 p0, p1, p2;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int d = 8 * b + e;
        const float v = (src && d < width) ? src[d] : 0.f;
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

template <int NQ, int PT, bool FT>
__global__ __launch_bounds__(fast_waves(NQ) * 64, fast_waves_per_simd(NQ)) void assign_fast_kernel(FastArgs a)
{
    constexpr int WAVES = fast_waves(NQ);
    constexpr int THREADS = WAVES * 64;
    constexpr int SU = fast_row_units(NQ);
    constexpr int TU = 32 * SU;  // units per tile
    constexpr int D8 = 8 * NQ;
    using M = Mma<float>;
    using G = TileGeom<FT>;
    constexpr int RG = G::RG;
    extern __shared__ __align__(16) uint4 lds4[];
    uint4 *ldsC = lds4;                                           // [tpc][TU]
    float *ldsH = reinterpret_cast<float *>(lds4 + (size_t)a.tpc * TU);  // [tpc*32] start values, (tile, group, register) order
    __shared__ int sh_next;
    __shared__ int sh_nf;
    __shared__ ftk_fault sh_faults[SMALLD_MAX_FAULTS];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int col = lane & 31;
    const int g = lane >> 5;
    const int D = a.D;
    const float cmax2 = (float)a.scal[0];
    const float cmax = sqrtf(cmax2);
    const bool resident = a.nch == 1;
    // wave-uniform event counters (scalar registers: counted with ballots)
    int n_injected = 0, n_detected = 0, n_corrected = 0, n_recomputed = 0;
    float worst_resid = 0.f;

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
            const int T = tile0 + tl;
            float h;
            if (!FT) {
                const int j = G::centroid(T, gg, r);
                h = j < a.K ? -a.hcn[j] : M::neg_inf();
            } else if (r < RG) {  // rows beyond K carry zeros and are dropped after the verification
                const int j = G::centroid(T, gg, r);
                h = j < a.K ? -a.hcn[j] : 0.f;
            } else {
                h = -a.chk_s[(T * 2 + gg) * 2];
            }
            ldsH[idx] = h;
        }
    };
    if (resident) {
        stage_chunk(0);
        __syncthreads();
    }

    // all the work on one unit of PT*32 points; blk = the point block the unit belongs to (fault addressing)
    auto process = [&](int unit, int blk) {
        const int64_t p0 = (int64_t)unit * (PT * 32);
        uint4 s0[PT][NQ], s1[PT][NQ], s2[PT][NQ];  // B fragments: (x0 | x0), (x1 | x1), (x0 | x2)
        float xn[PT];
        float tau[PT];          // checksum detection threshold of this lane's point
        float inv_tau[PT];
        int force_refine[PT];   // a tile of this point failed correction
        float rmax[PT];         // largest |residual| below the threshold over this point's tiles
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
            tau[pt] = (float)a.ft_coef * (sqrtf(s) * cmax + 0.5f * cmax2);
            inv_tau[pt] = 1.0f / tau[pt];
            force_refine[pt] = 0;
            rmax[pt] = 0.f;
            best[pt].m1 = best[pt].m2 = M::neg_inf();
            best[pt].t1 = 0;
        }

        // faults aimed at this point block
        int nf = 0;
        if (a.n_faults > 0) {
            if (tid == 0) sh_nf = 0;
            __syncthreads();
            for (int i = tid; i < a.n_faults; i += THREADS) {
                if ((int)a.faults[i].workgroup == blk) {
                    const int slot = atomicAdd(&sh_nf, 1);
                    if (slot < SMALLD_MAX_FAULTS) sh_faults[slot] = a.faults[i];
                }
            }
            __syncthreads();
            nf = min(sh_nf, SMALLD_MAX_FAULTS);
        }

        auto compute_tile = [&](auto inj_tag, const uint4 (&t0)[NQ], const uint4 (&t1)[NQ], const floatx16 &ci, int T) {
            constexpr bool INJ = decltype(inj_tag)::value;
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
                floatx16 acc = accs[pt];

                if constexpr (INJ) {  // fault injection (Section 2.1): flip one bit of one accumulator
                    for (int i = 0; i < nf; ++i) {
                        const ftk_fault f = sh_faults[i];
                        const int seq = (int)(f.tile % (unsigned)(a.tiles_total * PT));
                        if ((int)(f.wave % WAVES) == wave && seq == T * PT + pt) {
                            const bool me = lane == (int)(f.lane & 63);
                            const unsigned mask = 1u << (f.bit & 31);
                            const int reg = (int)(f.reg & 15);
#pragma unroll
                            for (int r = 0; r < 16; ++r) {
                                const unsigned bits = __float_as_uint(acc[r]);
                                acc[r] = (me && r == reg) ? __uint_as_float(bits ^ mask) : acc[r];
                            }
                            n_injected += (int)__popcll(__ballot(me));
                        }
                    }
                }

                if constexpr (FT) {
                    // verify: the 15 scores of this lane must add up to the carried checksum
                    float resid = sum15(acc) - acc[15];
                    bool bad = !(fabsf(resid) <= tau[pt]);
                    if (__builtin_expect(__any(bad), 0)) {
                        n_detected += (int)__popcll(__ballot(bad));
                        if (a.ft_mode >= FTK_FT_CORRECT) {
                            // locate with the e2 = 1..15 weighted sum (Section 4.1); its reference is formed
                            // here on demand, in fp32 on the vector units, from the point's row in memory
                            float s2w = 0.f;
#pragma unroll
                            for (int r = 0; r < RG; ++r) s2w = fmaf((float)(r + 1), acc[r], s2w);
                            int64_t p = p0 + pt * 32 + col;
                            if (p >= a.N) p = a.N - 1;
                            const float *xrow = a.X + p * D;
                            const float *v2 = a.chk_v2 + (size_t)(T * 2 + g) * D8;
                            float ref2 = -a.chk_s[(T * 2 + g) * 2 + 1];
#pragma unroll
                            for (int q = 0; q < 2 * NQ; ++q) {
                                const floatx4 xv = load_frag<float, true>(xrow, 4 * q, D);
                                const floatx4 vv = *reinterpret_cast<const floatx4 *>(v2 + 4 * q);
#pragma unroll
                                for (int e = 0; e < 4; ++e) ref2 = fmaf(xv[e], vv[e], ref2);
                            }
                            const float delta = resid;
                            const float fpos = (s2w - ref2) / delta;
                            const float rpos = rintf(fpos);
                            const bool finite = (__float_as_uint(delta) & 0x7f800000u) != 0x7f800000u;
                            // the location is trusted only when the error stands far enough above the
                            // rounding noise of the weighted sum; smaller detected errors are recomputed
                            bool ok = bad && finite && fabsf(delta) >= 32.f * tau[pt] && fabsf(fpos - rpos) < 0.25f &&
                                      rpos >= 1.f && rpos <= (float)RG;
                            const int rfix = ok ? (int)rpos - 1 : -1;
#pragma unroll
                            for (int r = 0; r < RG; ++r) acc[r] = (r == rfix) ? acc[r] - delta : acc[r];
                            ok = ok && (fabsf(sum15(acc) - acc[15]) <= tau[pt]);
                            n_corrected += (int)__popcll(__ballot(ok));
                            n_recomputed += (int)__popcll(__ballot(bad && !ok));
                            force_refine[pt] |= (bad && !ok) ? 1 : 0;
                        }
                        resid = bad ? 0.f : resid;  // statistics: fault-free residuals only
                    }
                    rmax[pt] = max2f(rmax[pt], fabsf(resid));
                    if (__builtin_expect(30 * (T + 1) > a.K, 0)) {  // last tile: rows beyond K carried zeros
#pragma unroll
                        for (int r = 0; r < RG; ++r)
                            acc[r] = (G::centroid(T, g, r) < a.K) ? acc[r] : M::neg_inf();
                    }
                }

                float tm;
                if constexpr (FT) {
                    tm = max3f(acc[0], acc[1], acc[2]);
#pragma unroll
                    for (int r = 3; r < 15; r += 2) tm = max3f(tm, acc[r], acc[r + 1]);
                } else {
                    tm = max2f(acc[0], acc[1]);
#pragma unroll
                    for (int r = 2; r < 16; r += 2) tm = max3f(tm, acc[r], acc[r + 1]);
                }
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
            auto sweep = [&](auto inj_tag) {
                if constexpr (NQ <= 2) {
                    // two operand register sets: the fetch of the next tile is in flight during the current one
                    uint4 t0A[NQ], t1A[NQ], t0B[NQ], t1B[NQ];
                    floatx16 ciA, ciB;
                    load_tile(0, t0A, t1A, ciA);
                    for (int t = 0; t < ntile; t += 2) {
                        load_tile(min(t + 1, ntile - 1), t0B, t1B, ciB);
                        compute_tile(inj_tag, t0A, t1A, ciA, tile0 + t);
                        load_tile(min(t + 2, ntile - 1), t0A, t1A, ciA);
                        if (t + 1 < ntile) compute_tile(inj_tag, t0B, t1B, ciB, tile0 + t + 1);
                    }
                } else {
                    // wide rows: one set (the registers are needed for the point fragments); the other
                    // wave of the SIMD covers the fetch
                    uint4 t0A[NQ], t1A[NQ];
                    floatx16 ciA;
                    for (int t = 0; t < ntile; ++t) {
                        load_tile(t, t0A, t1A, ciA);
                        compute_tile(inj_tag, t0A, t1A, ciA, tile0 + t);
                    }
                }
            };
            if (nf > 0)
                sweep(std::true_type{});
            else
                sweep(std::false_type{});
        }

        // ---- exact evaluation of the winning group; the two lanes of a point share its rows ----
#pragma unroll
        for (int pt = 0; pt < PT; ++pt) {
            if (FT) worst_resid = fmaxf(worst_resid, rmax[pt] * inv_tau[pt]);
            const int64_t p = p0 + pt * 32 + col;
            const bool live = p < a.N;
            const float *xrow = a.X + (live ? p : a.N - 1) * D;
            floatx4 xlo[NQ], xhi[NQ];
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                xlo[q] = load_frag<float, true>(xrow, 8 * q, D);
                xhi[q] = load_frag<float, true>(xrow, 8 * q + 4, D);
            }
            float bound = (float)a.band_coef * (sqrtf(xn[pt]) * cmax + 0.5f * cmax2);
            // strict FT: an error that stayed below the detection threshold left its mark in the
            // residual of its tile; the noise next to it is taken as at most half the threshold
            if (FT) bound += a.widen * (fmaxf(rmax[pt], __shfl_xor(rmax[pt], 32, 64)) + 0.5f * tau[pt]);
            const float om1 = __shfl_xor(best[pt].m1, 32, 64), om2 = __shfl_xor(best[pt].m2, 32, 64);
            const int ot1 = __shfl_xor(best[pt].t1, 32, 64);
            const bool mine_wins = best[pt].m1 > om1 || (best[pt].m1 == om1 && g == 0);
            const float thr = fmaxf(best[pt].m1, om1) - bound;
            const int gw = mine_wins ? g : 1 - g;
            const int Tw = mine_wins ? best[pt].t1 : ot1;
            const bool second = fminf(best[pt].m1, om1) >= thr;
            const int Ts = mine_wins ? ot1 : best[pt].t1;
            const bool over = fmaxf(best[pt].m2, om2) >= thr;
            const bool forced = (force_refine[pt] | __shfl_xor(force_refine[pt], 32, 64)) != 0;
            float dbest = __builtin_huge_valf();
            int jbest = 0x7fffffff;
            eval_rows<NQ, FT, false>(xlo, xhi, a.C, D, Tw, a.K, D, gw, 8 * g, dbest, jbest);
            if (__any(second)) {
                float d2 = dbest;
                int j2 = jbest;
                eval_rows<NQ, FT, false>(xlo, xhi, a.C, D, Ts, a.K, D, 1 - gw, 8 * g, d2, j2);
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
            // NaN scores, a third candidate, or a failed repair: exact recomputation
            worklist_push(live && g == 0 && (!(thr == thr) || over || forced), (int32_t)p, a.wl, a.wl_count);
        }
    };

    if (resident && a.n_faults == 0) {
        // Every centroid tile stays in LDS: the waves need no common step.  Each takes every
        // (grid * WAVES)-th unit - equal work per unit, so a fixed split balances, and a counter
        // drawn by every wave would cost one device-wide atomic per 64 points - and one wave's
        // exact settlement (a chain of memory latencies) runs under the matrix work of the others.
        for (int unit = (int)blockIdx.x * WAVES + wave; unit < a.nunits; unit += (int)gridDim.x * WAVES)
            process(unit, unit / WAVES);
    } else {
        // chunks are staged by the whole workgroup (and faults are listed per point block): its
        // waves walk the point blocks together
        int blk = blockIdx.x;
        while (blk < a.nblocks) {
            process(blk * WAVES + wave, blk);
            __syncthreads();
            if (tid == 0) sh_next = (int)gridDim.x + atomicAdd(a.wl_count + 1, 1);
            __syncthreads();
            blk = sh_next;
        }
    }

    // statistics (see the fp32 small-D kernel: few atomics, and only where something happened)
    if (a.stats && (FT || a.n_faults > 0)) {
        const int v[5] = {0, n_injected, n_detected, n_corrected, n_recomputed};
#pragma unroll
        for (int mask = 1; mask < 64; mask <<= 1) worst_resid = fmaxf(worst_resid, __shfl_xor(worst_resid, mask, 64));
        if (lane == 0) {
            unsigned long long *s = reinterpret_cast<unsigned long long *>(a.stats);
            if (FT && blockIdx.x == 0 && wave == 0) {  // every (point, tile, lane group) is verified once
                const long long units = (resident && a.n_faults == 0) ? a.nunits : (long long)a.nblocks * WAVES;
                atomicAdd(s, (unsigned long long)units * PT * 64 * a.tiles_total);
            }
            for (int i = 1; i < 5; ++i)
                if (v[i]) atomicAdd(s + i, (unsigned long long)v[i]);
            if (FT) {
                const unsigned long long mine = (unsigned long long)(fminf(worst_resid, 4000.f) * 1.0e6f);
                if (mine > *reinterpret_cast<volatile unsigned long long *>(s + 7)) atomicMax(s + 7, mine);
            }
        }
    }
}

bool fast_supported(ftk_dtype dtype, int D)
{
    return dtype == FTK_F32 && D <= 128 && D % 4 == 0;
}

size_t fast_split_bytes(ftk_dtype dtype, int D, int K)
{
    if (!fast_supported(dtype, D)) return 0;
    if (D > 32) return fast_wide_split_bytes(D, K);
    const int nq = (int)ceil_div(D, 8);
    // tiles of 30 centroids when checksums are on
    return (size_t)ceil_div(K, 30) * 32 * fast_row_units(nq) * sizeof(uint4);
}

// Detection threshold coefficient: that of the fp32 small-D tiles (15 scores against one
// checksum).  Each score is 3 * D/8 instructions here, but an instruction sums its 16 exact
// products at once and rounds once, so the residuals come out no larger than on the fp32 path
// (largest fault-free residual seen on the 2^20 x 8 and 2^21 x 32 workloads: 0.28 of the threshold).
static constexpr double FAST_FT_KAPPA = 1.0;
static double fast_ft_coef(int D)
{
    const double n = 15.0;
    return FAST_FT_KAPPA * Mma<float>::kEps * n * (std::sqrt(n) + std::sqrt((double)D + 4.0));
}

static int fast_tpc(int nq, int tiles_total)
{
    const int tile_bytes = 32 * fast_row_units(nq) * 16 + 32 * 4;
    // one workgroup per CU; all tiles resident if they fit, else equal chunks
    int tpc = (144 * 1024) / tile_bytes;
    if (tpc > tiles_total) tpc = tiles_total;
    return (int)ceil_div(tiles_total, ceil_div(tiles_total, tpc));
}

// The prologue (norms, their maximum, per-call state, checksum rows) is shared with the fp32 path;
// this fills what it and the geometry queries need.
void plan_fast(int64_t N, int D, int K, ftk_ft_mode ft, AssignPlan &p)
{
    if (D > 32) {
        plan_fast_wide(N, D, K, ft, p);
        return;
    }
    const bool FT = ft != FTK_FT_OFF;
    const int nq = (int)ceil_div(D, 8);
    p.variant = VAR_SMALLD;
    p.TM = 32;
    p.TN = 32;
    p.PT = fast_pt(nq);
    p.KT = 1;
    p.waves = fast_waves(nq);
    p.D8 = 8 * nq;
    p.DQ = nq;
    p.KC = 32;
    p.nkc = (int)ceil_div(K, FT ? 30 : 32);
    p.kch = fast_tpc(nq, p.nkc) * 32;
    p.hcn_pad_inf = !FT;
    p.points_per_wg = p.waves * p.PT * 32;
    p.workgroups = ceil_div(N, p.points_per_wg);
    p.grid = (int)(p.workgroups < 256 ? p.workgroups : 256);
    p.tiles_per_wave = p.nkc * p.PT;
    p.regs_per_tile = 16;
    p.lds_bytes = (size_t)(p.kch / 32) * (32 * fast_row_units(nq) * 16 + 32 * 4);
    p.ft_coef = fast_ft_coef(D);
    // two scores, each 3*nq instructions at 7 u of its magnitude, plus 2 u for the dropped
    // products and 2 u for the fp32 evaluation of the magnitude itself
    p.band_coef = 2.0 * (21.0 * nq + 4.0) * Mma<float>::kEps;
}

template <int NQ, bool FT>
static void launch_fast_t(FastArgs a, const AssignPlan &p, const float *chk_v1, hipStream_t st)
{
    constexpr int PT = fast_pt(NQ);
    const int rows = a.tiles_total * 32;
    hipLaunchKernelGGL((split_centroids_kernel<NQ, FT>), dim3((unsigned)ceil_div((int64_t)rows * NQ, 256)), dim3(256), 0,
                       st, a.C, chk_v1, a.D, a.K, a.tiles_total, const_cast<uint4 *>(a.csplit));
    hipLaunchKernelGGL((assign_fast_kernel<NQ, PT, FT>), dim3(p.grid), dim3(fast_waves(NQ) * 64), p.lds_bytes, st, a);
}

ftk_status launch_assign_fast(const AssignCall &c, const AssignPlan &p, const Workspace &w, hipStream_t st)
{
    if (c.D > 32) return launch_assign_fast_wide(c, p, w, st);
    if ((uintptr_t)c.X % 16 || (uintptr_t)c.C % 16) {
        set_error("the fast variant needs 16-byte aligned X and C");
        return FTK_EALIGN;
    }
    const bool FT = c.ft != FTK_FT_OFF;
    FastArgs a;
    a.X = (const float *)c.X;
    a.C = (const float *)c.C;
    a.hcn = (const float *)w.hcn;
    a.scal = w.scal;
    a.csplit = (const uint4 *)w.csplit;
    a.N = c.N;
    a.D = c.D;
    a.K = c.K;
    a.tiles_total = p.nkc;
    a.tpc = p.kch / 32;
    a.nch = (int)ceil_div(a.tiles_total, a.tpc);
    a.nblocks = (int)p.workgroups;
    a.nunits = (int)ceil_div(c.N, p.PT * 32);
    a.labels = c.labels;
    a.mindist = (float *)c.mindist;
    a.wl = w.wl;
    a.wl_count = w.wl_count;
    a.band_coef = p.band_coef;
    a.stats = c.stats;
    a.chk_v1 = (const float *)w.chk_v1;
    a.chk_v2 = (const float *)w.chk_v2;
    a.chk_s = (const float *)w.chk_s;
    a.faults = c.faults;
    a.n_faults = c.n_faults;
    a.ft_mode = (int)c.ft;
    a.ft_coef = p.ft_coef;
    a.widen = c.ft == FTK_FT_STRICT ? 1.0f : 0.0f;
    const float *v1 = (const float *)w.chk_v1;
#define FTK_LAUNCH_FAST(NQV)                              \
    do {                                                  \
        if (FT) launch_fast_t<NQV, true>(a, p, v1, st);   \
        else launch_fast_t<NQV, false>(a, p, v1, st);     \
    } while (0)
    switch (p.DQ) {
    case 1: FTK_LAUNCH_FAST(1); break;
    case 2: FTK_LAUNCH_FAST(2); break;
    case 3: FTK_LAUNCH_FAST(3); break;
    default: FTK_LAUNCH_FAST(4); break;
    }
#undef FTK_LAUNCH_FAST
    FTK_TRY_HIP(hipGetLastError());
    return FTK_OK;
}

}  // namespace ftk
