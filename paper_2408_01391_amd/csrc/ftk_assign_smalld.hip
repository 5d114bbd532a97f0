// Small-D assignment kernel (fp32, D <= 32, rows 16-byte aligned), with optional checksums.
//
// With few features the contraction per output tile is only D/2 matrix instructions, so the
// per-element epilogue work decides the speed (the paper notes the same for small feature
// counts in Section 5.1: data movement and the row-wise reduction become the critical part;
// on this hardware fp32 matrix and vector instructions do not overlap, so every epilogue
// instruction adds to the matrix time).  This variant therefore
//   * keeps the point fragments (B operand) in registers for the whole sweep over K: X is read
//     once, straight from HBM with 16-byte coalesced loads, and never goes through LDS;
//   * stages centroids (A operand) in LDS together with their -||c||^2/2 terms laid out in
//     accumulator order, so each tile starts from four broadcast 16-byte LDS reads;
//   * reduces every 32x32 output tile to ONE maximum per lane with v_max3 (half an op per
//     score) and keeps only the best tile, its maximum and the runner-up tile maximum;
//   * after the sweep re-evaluates the winning group of 16 centroids in direct-difference form
//     (the two lanes of a point share the rows), which yields the exact arg-min inside the
//     group, resolves near-ties the cancelling expanded form cannot order, and gives an
//     accurate minimum distance;
//   * evaluates a second group when the other lane's best tile is inside the rounding bound; a
//     third candidate sends the point to the refine kernel.  With strict fault tolerance, where
//     the bound is wider and a few per cent of the points are ambiguous, such points are instead
//     collected per workgroup and swept a second time at the end of the kernel with the two best
//     tiles of each lane on record (see the kernel).
//
// Fault tolerance (Sections 2.3, 4): with FT on, every tile carries its own checksum row.  A
// tile then holds 30 centroids; register 15 of each lane group belongs to a virtual centroid
// "sum of the group's 15 centroids" (the Y e1 encoding, prepared by a prologue kernel), so the
// matrix instructions deliver x.(sum c) - sum ||c||^2/2 next to the 15 scores it must equal.
// After the tile's instructions (and the injection hook) each lane adds its 15 scores and
// compares; a mismatch above the threshold is located with the e2 = 1..15 weighted sum
// (Section 4.1), corrected by subtracting the error, and re-verified before the maximum reads
// the tile.  If the location does not decode, the point is handed to the refine kernel, which
// recomputes it without the matrix path.
#include <cmath>
#include <type_traits>

#include "ftk_internal.h"
#include "ftk_mma.h"
#include "ftk_smalld.h"

namespace ftk {

struct SmallArgs {
    const float *X;
    const float *C;
    const float *hcn;    // half squared norms; beyond K: +inf (FT off) or unused (FT on)
    const double *scal;  // scal[0] = max_j ||c_j||^2
    int64_t N;
    int D, K;
    int tpc;          // tiles staged in LDS at a time
    int nch;          // chunks
    int tiles_total;  // ceil(K / centroids-per-tile)
    int nblocks;      // point blocks (waves*PT*32 points each)
    int32_t *labels;
    float *mindist;
    int32_t *wl;        // work-list of the refine kernel (point indices)
    int32_t *wl_count;  // [0] its length, [1] block counter
    int defer;          // 1 = collect ambiguous points per workgroup and sweep them a second time (when
                        // every tile is LDS-resident); 0 = evaluate the other lane's best group where it
                        // turns up and leave third candidates to the refine kernel
    ftk_ft_stats *stats;
    double band_coef;
    // fault tolerance / injection
    const float *chk_v1;  // [tiles_total*2][D8] plain checksum rows per (tile, lane group)
    const float *chk_v2;  // [tiles_total*2][D8] weighted (1..15) checksum rows
    const float *chk_s;   // [tiles_total*2][2]  matching sums of the half norms
    const ftk_fault *faults;
    int n_faults;
    int ft_mode;
    double ft_coef;       // detection threshold = ft_coef * (||x|| max||c|| + max||c||^2/2)
    float widen;          // 1 in strict mode (the ambiguity band grows by the threshold), else 0
};

// waves per workgroup sharing one staged centroid chunk (measured: 8 beats 4 for every D <= 32,
// even where the exact re-evaluation then spills a few registers)
static constexpr int smalld_waves(int nq, bool ft) { return nq <= 4 ? 8 : 4; }
// waves per SIMD the register budget is sized for (the second launch-bound is waves per
// execution unit): two resident workgroups of eight waves need four
static constexpr int smalld_min_wgs(int nq, bool ft) { return nq <= 1 ? 4 : 2; }

template <int NQ, int PT, bool FT>
__global__ __launch_bounds__(smalld_waves(NQ, FT) * 64, smalld_min_wgs(NQ, FT)) void assign_smalld_kernel(SmallArgs a)
{
    constexpr int SMALLD_WAVES = smalld_waves(NQ, FT);
    constexpr int SMALLD_THREADS = SMALLD_WAVES * 64;
    using M = Mma<float>;
    using G = TileGeom<FT>;
    constexpr int SW = 8 * NQ + 4;      // LDS row stride in floats (16 bytes of padding)
    constexpr int TS = 32 * SW + 4;     // LDS tile stride: 16 more bytes so that lanes reading rows
                                        // of different tiles (exact re-evaluation) spread over banks
    constexpr int RG = G::RG;
    constexpr int D8 = 8 * NQ;
    extern __shared__ __align__(16) float lds[];
    float *ldsC = lds;                          // [tpc][TS]
    float *ldsH = lds + (size_t)a.tpc * TS;     // [tpc*32] accumulator start values, (tile, group, register) order
    __shared__ int sh_next;
    __shared__ int sh_nf;
    __shared__ int sh_wlcnt;
    __shared__ int32_t sh_wl[SMALLD_LIST_CAP];
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
    // deferred mode (every tile resident): ambiguous points are not settled where they turn up but
    // collected per workgroup and swept once more at the end, see below
    const bool defer = a.defer != 0 && resident;
    // wave-uniform event counters (scalar registers: counted with ballots)
    int n_injected = 0, n_detected = 0, n_corrected = 0, n_recomputed = 0;
    float worst_resid = 0.f;  // largest fault-free residual seen by this lane, in units of its threshold

    // slots a wave reserved but could not use stay marked
    for (int i = tid; i < SMALLD_LIST_CAP; i += SMALLD_THREADS) sh_wl[i] = -1;
    if (tid == 0) sh_wlcnt = 0;

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

    // stage tiles [ch*tpc, (ch+1)*tpc) into LDS: centroid rows (and checksum rows) plus the
    // accumulator start values.  A thread keeps its 16-byte piece of the row and walks the rows
    // with a fixed stride; the loads are branch-free (clamped addresses, zeros selected
    // afterwards) and issued up to eight at a time: a chunk costs a few memory round trips, not
    // one per row, which matters where the chunks change inside the sweep (K * D beyond the LDS).
    auto stage_chunk = [&](int ch) {
        constexpr int PPR = 2 * NQ;                    // 16-byte pieces per row
        constexpr int RSTEP = SMALLD_THREADS / PPR;    // rows per pass of the workgroup (left-over threads idle)
        constexpr int SU = NQ == 1 ? 4 : 8;            // loads in flight (the 128-register variant has room for four)
        const int rows = a.tpc * 32;
        const int st_pc = tid % PPR, st_r0 = tid / PPR;
        if (st_r0 < RSTEP) {
            for (int rb = st_r0; rb < rows; rb += SU * RSTEP) {
                floatx4 f[SU];
#pragma unroll
                for (int u = 0; u < SU; ++u) {
                    const int rrow = min(rb + u * RSTEP, rows - 1);
                    const int tl = rrow >> 5, lr = rrow & 31;
                    const int T = ch * a.tpc + tl;
                    const int gg = (lr >> 2) & 1, r = (lr >> 3) * 4 + (lr & 3);
                    const bool chk = FT && r >= RG;  // a checksum row (D8 wide), else a centroid row (D wide)
                    const int j = G::centroid(T, gg, r);
                    const int width = chk ? D8 : D;
                    const bool keep = (chk ? T < a.tiles_total : j < a.K) && 4 * st_pc < width;
                    const float *src = chk ? a.chk_v1 + (size_t)(min(T, a.tiles_total - 1) * 2 + gg) * D8
                                           : a.C + (size_t)min(j, a.K - 1) * D;
                    const floatx4 v = *reinterpret_cast<const floatx4 *>(src + min(4 * st_pc, width - 4));
#pragma unroll
                    for (int e = 0; e < 4; ++e) f[u][e] = keep ? v[e] : 0.f;
                }
#pragma unroll
                for (int u = 0; u < SU; ++u) {
                    const int rrow = rb + u * RSTEP;
                    if (rrow < rows)
                        *reinterpret_cast<floatx4 *>(ldsC + (size_t)(rrow >> 5) * TS + (rrow & 31) * SW + 4 * st_pc) = f[u];
                }
            }
        }
        for (int idx = tid; idx < rows; idx += SMALLD_THREADS) {
            const int tl = idx >> 5, gg = (idx >> 4) & 1, r = idx & 15;
            const int T = ch * a.tpc + tl;
            float h;
            if (!FT) {
                h = -a.hcn[G::centroid(T, gg, r)];
            } else if (r < RG) {
                const int j = G::centroid(T, gg, r);
                h = j < a.K ? -a.hcn[j] : 0.f;
            } else {
                h = T < a.tiles_total ? -a.chk_s[(T * 2 + gg) * 2] : 0.f;
            }
            ldsH[idx] = h;
        }
    };
    if (resident) stage_chunk(0);
    __syncthreads();

    // Blocks of SMALLD_WAVES units (PT*32 points per wave).  While chunks have to be staged (or
    // faults are listed per block) the waves of a workgroup walk the blocks in step and draw them
    // from an atomic counter, one draw per block.  With every tile resident nothing ties the
    // waves together: each then takes every gridDim-th block on its own, without barriers, so the
    // memory latencies at the start and the end of a block (point rows, exact re-evaluation) of
    // one wave run under the matrix work of the others.  (A counter drawn per wave instead would
    // put one device-wide atomic on the same word per 64 points, which costs more than it saves.)
    //
    // Deferred mode adds a SECOND ROUND after the blocks: the points the workgroup's waves found
    // ambiguous (another tile maximum inside the rounding bound - with strict fault tolerance a
    // few per cent of all points) sit in the LDS list; wave w takes entries [w*PT*32, (w+1)*PT*32)
    // and sweeps the resident tiles once more for them, this time also recording which tiles held
    // the two best maxima of each lane, and evaluates up to four candidate groups exactly.  The
    // extra record costs four vector instructions per tile, which is why the first round does not
    // keep it; evaluating a second group where it turns up would make a whole wave pay for one
    // lane, and sending every such point to the refine kernel (all K distances) costs far more.
    // one unit of work of a wave: PT*32 points starting at p0 of `npoints` (first round: points of
    // X; second round, R2: entries of the workgroup's list), swept over all tiles and settled
    auto process = [&](auto r2_tag, int64_t p0, int64_t npoints, int blk) {
        constexpr bool R2 = decltype(r2_tag)::value;
        floatx4 xf[PT][NQ];
        float xn[PT];
        float tau[PT];          // checksum detection threshold of this lane's point
        float inv_tau[PT];
        int force_refine[PT];   // a tile of this point failed correction (int, not bool: a bool
                                // array updated inside the rare branch lost its value when compiled)
        float rmax[PT];         // largest |residual| below the threshold over this point's tiles
        TileBest best[PT];
        float m3[R2 ? PT : 1];  // second round: third-best tile maximum and the runner-up's tile
        int t2[R2 ? PT : 1];
        int pidx[PT];           // the point this lane works on (-1: none)
#pragma unroll
        for (int pt = 0; pt < PT; ++pt) {
            int64_t p = p0 + pt * 32 + col;
            if (p >= npoints) p = npoints - 1;
            if (R2) p = sh_wl[p];
            pidx[pt] = (int)p;
            const float *xrow = a.X + (p < 0 ? 0 : p) * D;
            float s = 0.f;
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                xf[pt][q] = load_frag<float, true>(xrow, 8 * q + 4 * g, D);
#pragma unroll
                for (int e = 0; e < 4; ++e) s = fmaf(xf[pt][q][e], xf[pt][q][e], s);
            }
            xn[pt] = s + __shfl_xor(s, 32, 64);
            tau[pt] = (float)a.ft_coef * (sqrtf(xn[pt]) * cmax + 0.5f * cmax2);
            inv_tau[pt] = 1.0f / tau[pt];
            force_refine[pt] = 0;
            rmax[pt] = 0.f;
            best[pt].m1 = best[pt].m2 = M::neg_inf();
            best[pt].t1 = 0;
            if constexpr (R2) {
                m3[pt] = M::neg_inf();
                t2[pt] = 0;
            }
        }

        // faults aimed at this point block (descriptors address the blocks of the first round)
        int nf = 0;
        if (!R2 && a.n_faults > 0) {
            if (tid == 0) sh_nf = 0;
            __syncthreads();
            for (int i = tid; i < a.n_faults; i += SMALLD_THREADS) {
                if ((int)a.faults[i].workgroup == blk) {
                    const int slot = atomicAdd(&sh_nf, 1);
                    if (slot < SMALLD_MAX_FAULTS) sh_faults[slot] = a.faults[i];
                }
            }
            __syncthreads();
            nf = min(sh_nf, SMALLD_MAX_FAULTS);
        }

        // one output tile: contraction, (injection, verification,) tile maximum, running best
        auto compute_tile = [&](auto inj_tag, auto round2_tag, const floatx4 (&av)[NQ], const floatx16 &ci, int T) {
            constexpr bool INJ = decltype(inj_tag)::value;
            constexpr bool ROUND2 = decltype(round2_tag)::value;
            // all matrix instructions of the tile first: the PT accumulator chains are independent
            // and interleave on the matrix pipe; verification and reduction follow per point tile
            floatx16 accs[PT];
#pragma unroll
            for (int pt = 0; pt < PT; ++pt) accs[pt] = ci;
#pragma unroll
            for (int q = 0; q < NQ; ++q)
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int pt = 0; pt < PT; ++pt) accs[pt] = M::mma(av[q][e], xf[pt][q][e], accs[pt]);
#pragma unroll
            for (int pt = 0; pt < PT; ++pt) {
                floatx16 acc = accs[pt];

                if constexpr (INJ) {  // fault injection (Section 2.1): flip one bit of one accumulator
                    for (int i = 0; i < nf; ++i) {
                        const ftk_fault f = sh_faults[i];
                        const int seq = (int)(f.tile % (unsigned)(a.tiles_total * PT));
                        if ((int)(f.wave % SMALLD_WAVES) == wave && seq == T * PT + pt) {
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
                            // locate with the e2 = 1..15 weighted sum; the weighted reference is
                            // formed here on demand from the weighted checksum row
                            float s2 = 0.f;
#pragma unroll
                            for (int r = 0; r < RG; ++r) s2 = fmaf((float)(r + 1), acc[r], s2);
                            float ref2 = 0.f;
                            if (T < a.tiles_total) {
                                const float *v2 = a.chk_v2 + (size_t)(T * 2 + g) * D8;
                                ref2 = -a.chk_s[(T * 2 + g) * 2 + 1];
#pragma unroll
                                for (int q = 0; q < NQ; ++q) {
                                    const floatx4 vo = *reinterpret_cast<const floatx4 *>(v2 + 8 * q + 4 * g);
                                    const floatx4 vp = *reinterpret_cast<const floatx4 *>(v2 + 8 * q + 4 * (1 - g));
#pragma unroll
                                    for (int e = 0; e < 4; ++e) {
                                        const float xo = xf[pt][q][e];
                                        const float xp = __shfl_xor(xo, 32, 64);
                                        ref2 = fmaf(xo, vo[e], ref2);
                                        ref2 = fmaf(xp, vp[e], ref2);
                                    }
                                }
                            }
                            const float delta = resid;
                            const float fpos = (s2 - ref2) / delta;
                            const float rpos = rintf(fpos);
                            const bool finite = (__float_as_uint(delta) & 0x7f800000u) != 0x7f800000u;
                            // The location is only trusted when the error stands far enough above the
                            // rounding noise of the weighted sum (weights up to 15) for the quotient to be
                            // accurate to a quarter; smaller detected errors are recomputed instead.  (After
                            // subtracting delta the plain checksum matches wherever it was subtracted, so a
                            // wrong location would go unnoticed.)
                            bool ok = bad && finite && fabsf(delta) >= 32.f * tau[pt] && fabsf(fpos - rpos) < 0.25f &&
                                      rpos >= 1.f && rpos <= (float)RG;
                            const int rfix = ok ? (int)rpos - 1 : -1;
#pragma unroll
                            for (int r = 0; r < RG; ++r) acc[r] = (r == rfix) ? acc[r] - delta : acc[r];
                            ok = ok && (fabsf(sum15(acc) - acc[15]) <= tau[pt]);
                            n_corrected += (int)__popcll(__ballot(ok));
                            // not decodable (error in the checksum register itself, several errors,
                            // Inf/NaN): the point is recomputed outside the matrix path
                            n_recomputed += (int)__popcll(__ballot(bad && !ok));
                            force_refine[pt] |= (bad && !ok) ? 1 : 0;
                        }
                        resid = bad ? 0.f : resid;  // statistics: fault-free residuals only
                    }
                    rmax[pt] = max2f(rmax[pt], fabsf(resid));  // one instruction; NaN went the branch above
                    if (__builtin_expect(30 * (T + 1) > a.K, 0)) {  // last tile: rows beyond K carried zeros, now drop them
#pragma unroll
                        for (int r = 0; r < RG; ++r)
                            acc[r] = (G::centroid(T, g, r) < a.K) ? acc[r] : M::neg_inf();
                    }
                }

                float tm;
                if constexpr (FT) {  // 15 scores
                    tm = max3f(acc[0], acc[1], acc[2]);
#pragma unroll
                    for (int r = 3; r < 15; r += 2) tm = max3f(tm, acc[r], acc[r + 1]);
                } else {             // 16 scores
                    tm = max2f(acc[0], acc[1]);
#pragma unroll
                    for (int r = 2; r < 16; r += 2) tm = max3f(tm, acc[r], acc[r + 1]);
                }
                const float m1 = best[pt].m1, m2 = best[pt].m2;
                const int t1 = best[pt].t1;
                const bool c = tm > m1;
                if constexpr (ROUND2) {  // sorted insert into (m1 >= m2 >= m3), tiles of the first two
                    const bool c2 = tm > m2;
                    m3[pt] = __builtin_amdgcn_fmed3f(m2, m3[pt], tm);
                    const int t2n = c2 ? T : t2[pt];
                    t2[pt] = c ? t1 : t2n;
                }
                best[pt].m2 = __builtin_amdgcn_fmed3f(m1, m2, tm);
                best[pt].t1 = c ? T : t1;
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
            // two operand register sets: the fetch of the next tile is in flight while the
            // current one is multiplied; the injection hook is compiled in only when faults are
            // listed for this block, so the common sweep has no per-tile branch for it
            auto sweep = [&](auto inj_tag, auto round2_tag) {
                floatx4 avA[NQ], avB[NQ];
                floatx16 ciA, ciB;
                load_tile(0, avA, ciA);
                for (int t = 0; t < ntile; t += 2) {
                    load_tile(min(t + 1, ntile - 1), avB, ciB);
                    compute_tile(inj_tag, round2_tag, avA, ciA, tile0 + t);
                    load_tile(min(t + 2, ntile - 1), avA, ciA);
                    if (t + 1 < ntile) compute_tile(inj_tag, round2_tag, avB, ciB, tile0 + t + 1);
                }
            };
            if (R2)
                sweep(std::false_type{}, std::true_type{});
            else if (nf > 0)
                sweep(std::true_type{}, std::false_type{});
            else
                sweep(std::false_type{}, std::false_type{});
        }

        // ---- exact evaluation of the winning group; the two lanes of a point share its rows ----
#pragma unroll
        for (int pt = 0; pt < PT; ++pt) {
            if (FT) worst_resid = fmaxf(worst_resid, rmax[pt] * inv_tau[pt]);
            const int64_t slot = p0 + pt * 32 + col;
            const int64_t p = pidx[pt];
            const bool live = slot < npoints && p >= 0;
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
            // scores inside `bound` of each other cannot be ordered: rounding of the expanded
            // form, plus (strict FT) an undetected error below the detection threshold
            float bound = (float)a.band_coef * (sqrtf(xn[pt]) * cmax + 0.5f * cmax2);
            // strict FT: an error that stayed below the detection threshold left its mark in the
            // residual of its tile, |error| <= |residual| + rounding noise; the noise is taken as at
            // most half the threshold (fault-free residuals reach about 0.3 of it), the residual as
            // the largest either lane of the point saw
            if (FT) bound += a.widen * (fmaxf(rmax[pt], __shfl_xor(rmax[pt], 32, 64)) + 0.5f * tau[pt]);
            const float om1 = __shfl_xor(best[pt].m1, 32, 64), om2 = __shfl_xor(best[pt].m2, 32, 64);
            const int ot1 = __shfl_xor(best[pt].t1, 32, 64);
            const bool mine_wins = best[pt].m1 > om1 || (best[pt].m1 == om1 && g == 0);
            const float thr = fmaxf(best[pt].m1, om1) - bound;
            // the group holding the best tile maximum (gw = its lane group)
            const int gw = mine_wins ? g : 1 - g;
            const int Tw = mine_wins ? best[pt].t1 : ot1;
            const bool forced = (force_refine[pt] | __shfl_xor(force_refine[pt], 32, 64)) != 0;
            float dbest = __builtin_huge_valf();
            int jbest = 0x7fffffff;
            // one group of 16 (15) rows, split between the two lanes of the point; `take` = whether
            // this point counts the group (the evaluation itself runs for the whole wave)
            auto eval_group = [&](int T, int gsel, bool take) {
                float d2 = dbest;
                int j2 = jbest;
                if (resident)
                    eval_rows<NQ, FT, true>(xlo, xhi, ldsC + T * TS, SW, T, a.K, D, gsel, 8 * g, d2, j2);
                else
                    eval_rows<NQ, FT, false>(xlo, xhi, a.C, D, T, a.K, D, gsel, 8 * g, d2, j2);
                dbest = take ? d2 : dbest;
                jbest = take ? j2 : jbest;
            };
            eval_group(Tw, gw, true);
            // another tile maximum inside the bound: the best tile of the losing lane ...
            const bool cand_b = fminf(best[pt].m1, om1) >= thr;
            const int Tb = mine_wins ? ot1 : best[pt].t1;
            bool unsettled;
            if constexpr (!R2) {
                // ... evaluated here unless ambiguous points are deferred; a runner-up tile of either
                // lane is not on record in the first round
                if (!defer && __any(cand_b)) eval_group(Tb, 1 - gw, cand_b);
                unsettled = (defer && cand_b) || fmaxf(best[pt].m2, om2) >= thr;
            } else {
                // ... and the runner-up tiles of the winning and of the losing lane, each only if
                // some point of the wave needs it
                const int ot2 = __shfl_xor(t2[pt], 32, 64);
                const float wm2 = mine_wins ? best[pt].m2 : om2, lm2 = mine_wins ? om2 : best[pt].m2;
                const bool cand_c = wm2 >= thr, cand_d = lm2 >= thr;
                const int Tc = mine_wins ? t2[pt] : ot2, Td = mine_wins ? ot2 : t2[pt];
                if (__any(cand_b)) eval_group(Tb, 1 - gw, cand_b);
                if (__any(cand_c)) eval_group(Tc, gw, cand_c);
                if (__any(cand_d)) eval_group(Td, 1 - gw, cand_d);
                // a third tile of either lane inside the bound: left to the refine kernel
                unsettled = fmaxf(m3[pt], __shfl_xor(m3[pt], 32, 64)) >= thr;
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
            // NaN scores, more candidates than are on record, or a failed repair: exact recomputation
            const bool need = live && g == 0 && (!(thr == thr) || unsettled || forced);
            if (R2)
                worklist_push(need, (int32_t)p, a.wl, a.wl_count);
            else
                block_list_push(need, (int32_t)p, sh_wl, &sh_wlcnt, a.wl, a.wl_count);
        }
    };

    int blk = blockIdx.x;
    while (blk < a.nblocks) {
        process(std::false_type{}, ((int64_t)blk * SMALLD_WAVES + wave) * (PT * 32), a.N, blk);
        if (resident && a.n_faults == 0) {
            blk += (int)gridDim.x;
            continue;
        }
        __syncthreads();
        if (tid == 0) sh_next = (int)gridDim.x + atomicAdd(a.wl_count + 1, 1);
        __syncthreads();
        blk = sh_next;
    }
    if (defer) {
        __syncthreads();  // every wave is through its blocks: the list is complete
        const int nlist = min(sh_wlcnt, SMALLD_LIST_CAP);
        // Units of PT*32 entries go to every other wave: the even ones in even-numbered
        // workgroups, the odd ones in odd-numbered ones, so that the few sweeping waves of two
        // workgroups sharing a CU (consecutive waves sit on consecutive SIMDs) tend to land on
        // different SIMDs instead of sharing two of the four.
        if ((wave & 1) == ((int)blockIdx.x & 1))
            for (int unit = wave >> 1; unit * (PT * 32) < nlist; unit += SMALLD_WAVES / 2)
                process(std::true_type{}, (int64_t)unit * (PT * 32), (int64_t)nlist, 0);
    }

    if (!defer) {  // hand the collected work-list entries over to the refine kernel
        __syncthreads();
        const int n = min(sh_wlcnt, SMALLD_LIST_CAP);
        for (int i0 = 0; i0 < n; i0 += SMALLD_THREADS) {
            const int i = i0 + tid;
            const int32_t v = i < n ? sh_wl[i] : -1;
            worklist_push(v >= 0, v, a.wl, a.wl_count);
        }
    }

    // Statistics.  Thousands of waves adding to the same few words would keep the memory system
    // busy long after the last wave has ended, so: the number of comparisons made is known in
    // advance and added once; the other counters are touched only when non-zero (i.e. when a
    // fault was seen); the residual maximum is read first and raised only by a wave that exceeds it.
    if (a.stats && (FT || a.n_faults > 0)) {
        const int v[5] = {0, n_injected, n_detected, n_corrected, n_recomputed};
#pragma unroll
        for (int mask = 1; mask < 64; mask <<= 1) worst_resid = fmaxf(worst_resid, __shfl_xor(worst_resid, mask, 64));
        if (lane == 0) {
            unsigned long long *s = reinterpret_cast<unsigned long long *>(a.stats);
            if (FT && blockIdx.x == 0 && wave == 0)  // every (point, tile, lane group) is verified once
                atomicAdd(s, (unsigned long long)a.nblocks * SMALLD_WAVES * PT * 64 * a.tiles_total);
            for (int i = 1; i < 5; ++i)
                if (v[i]) atomicAdd(s + i, (unsigned long long)v[i]);
            if (FT) {
                const unsigned long long mine = (unsigned long long)(fminf(worst_resid, 4000.f) * 1.0e6f);
                if (mine > *reinterpret_cast<volatile unsigned long long *>(s + 7)) atomicMax(s + 7, mine);
            }
        }
    }
}

// Checksum rows of the small-D tiles (FT on): for tile T and lane group g, over the group's 15
// centroids j = 30T + 15g + r (those below K):
//   v1[d] = sum_r c_{j,d}, v2[d] = sum_r (r+1) c_{j,d}   (the Y e1 / Y e2 encodings, Section 4.1)
// in double, rounded once; and the matching sums of the half squared norms.
__global__ __launch_bounds__(64) void smalld_checksum_kernel(const float *C, const float *hcn, int D, int D8,
                                                             int K, float *v1, float *v2, float *cs)
{
    const int tg = blockIdx.x;  // T*2 + g
    const int j0 = 30 * (tg >> 1) + 15 * (tg & 1);
    for (int d = threadIdx.x; d < D8; d += blockDim.x) {
        double s1 = 0.0, s2 = 0.0;
        if (d < D) {
            for (int r = 0; r < 15 && j0 + r < K; ++r) {
                const double v = (double)C[(size_t)(j0 + r) * D + d];
                s1 += v;
                s2 = fma((double)(r + 1), v, s2);
            }
        }
        v1[(size_t)tg * D8 + d] = (float)s1;
        v2[(size_t)tg * D8 + d] = (float)s2;
    }
    if (threadIdx.x == 0) {
        double h1 = 0.0, h2 = 0.0;
        for (int r = 0; r < 15 && j0 + r < K; ++r) {
            const double h = (double)hcn[j0 + r];
            h1 += h;
            h2 = fma((double)(r + 1), h, h2);
        }
        cs[2 * tg] = (float)h1;
        cs[2 * tg + 1] = (float)h2;
    }
}

ftk_status launch_smalld_checksums(const AssignCall &c, const AssignPlan &p, const Workspace &w, hipStream_t st)
{
    const int tiles_total = (int)ceil_div(c.K, 30);
    hipLaunchKernelGGL(smalld_checksum_kernel, dim3(tiles_total * 2), dim3(64), 0, st, (const float *)c.C,
                       (const float *)w.hcn, c.D, p.D8, c.K, (float *)w.chk_v1, (float *)w.chk_v2,
                       (float *)w.chk_s);
    FTK_TRY_HIP(hipGetLastError());
    return FTK_OK;
}

bool smalld_supported(ftk_dtype dtype, int D, int K)
{
    (void)K;
    return dtype == FTK_F32 && D <= 32 && D % 4 == 0;
}

// Detection threshold coefficient: the residual "15 scores minus carried checksum" is pure
// rounding noise when no fault occurred.  With n = 15 terms of magnitude up to
// B = ||x|| max||c|| + max||c||^2/2, the vector sum, the checksum product (magnitude up to n B)
// and the scores themselves each contribute about u B n (sqrt(n) + sqrt(D)) in the worst
// realistic alignment; KAPPA is the safety factor on top (calibrated so that the largest
// fault-free residual seen on the five workloads stays below half the threshold).
static constexpr double SMALLD_FT_KAPPA = 1.0;
static double smalld_ft_coef(int D)
{
    const double n = 15.0;
    return SMALLD_FT_KAPPA * Mma<float>::kEps * n * (std::sqrt(n) + std::sqrt((double)D + 4.0));
}

void plan_smalld(int64_t N, int D, int K, ftk_ft_mode ft, AssignPlan &p)
{
    const bool FT = ft != FTK_FT_OFF;
    p.variant = VAR_SMALLD;
    p.TM = 32;
    p.TN = 32;
    p.D8 = (int)ceil_div(D, 8) * 8;
    // point tiles per wave: two; four for wide rows when there are points enough to keep every
    // workgroup busy with blocks of 1024 (each centroid fragment then feeds twice the matrix work:
    // c5 -2 %)
    p.PT = (p.D8 >= 24 && N >= (1 << 19)) ? 4 : 2;
    p.KT = 1;
    p.waves = smalld_waves(p.D8 / 8, FT);
    const int SW = p.D8 + 4;
    const int tile_bytes = (32 * SW + 4) * 4 + 32 * 4;
    const int tiles_total = (int)ceil_div(K, FT ? 30 : 32);
    // chunk: as many tiles as fit the LDS share of a workgroup, all of them if possible.  D <= 8
    // runs two workgroups per CU (72 KB each); wider rows need more than 128 registers per lane,
    // so one workgroup has the CU to itself and can stage nearly all of its 160 KB (156 KB: 1024
    // centroids of 32 features stay resident)
    int tpc = ((p.D8 <= 8 ? 72 : 156) * 1024) / tile_bytes;
    if (tpc > tiles_total) tpc = tiles_total;
    // equal chunks: the same number of passes, but no short last chunk paying a full stage
    tpc = (int)ceil_div(tiles_total, ceil_div(tiles_total, tpc));
    p.kch = tpc * 32;
    p.KC = tpc * 32;
    p.nkc = (int)ceil_div(tiles_total, tpc);
    p.DQ = p.D8 / 8;
    p.points_per_wg = p.waves * p.PT * 32;
    p.workgroups = ceil_div(N, p.points_per_wg);
    p.lds_bytes = (size_t)tpc * tile_bytes;
    int resident_wgs = (int)(160 * 1024 / (p.lds_bytes + 2048));
    if (resident_wgs > 2) resident_wgs = 2;
    if (resident_wgs < 1) resident_wgs = 1;
    const int64_t cap = 256LL * resident_wgs;
    p.grid = (int)(p.workgroups < cap ? p.workgroups : cap);
    p.tiles_per_wave = tiles_total * p.PT;
    p.regs_per_tile = 16;
    p.hcn_pad_inf = !FT;
    p.ft_coef = smalld_ft_coef(D);
    // two scores, each a chain of D8 fused multiply-adds rounded to nearest (see the generic variant)
    p.band_coef = 2.0 * (p.D8 + 4) * Mma<float>::kEps;
}

template <int NQ>
static void launch_smalld_t(const SmallArgs &a, const AssignPlan &p, bool ft, hipStream_t st)
{
    if constexpr (NQ >= 3) {
        if (p.PT == 4) {
            if (ft)
                hipLaunchKernelGGL((assign_smalld_kernel<NQ, 4, true>), dim3(p.grid), dim3(smalld_waves(NQ, true) * 64), p.lds_bytes, st, a);
            else
                hipLaunchKernelGGL((assign_smalld_kernel<NQ, 4, false>), dim3(p.grid), dim3(smalld_waves(NQ, false) * 64), p.lds_bytes, st, a);
            return;
        }
    }
    if (ft)
        hipLaunchKernelGGL((assign_smalld_kernel<NQ, 2, true>), dim3(p.grid), dim3(smalld_waves(NQ, true) * 64), p.lds_bytes, st, a);
    else
        hipLaunchKernelGGL((assign_smalld_kernel<NQ, 2, false>), dim3(p.grid), dim3(smalld_waves(NQ, false) * 64), p.lds_bytes, st, a);
}

ftk_status launch_assign_smalld(const AssignCall &c, const AssignPlan &p, const Workspace &w, hipStream_t st)
{
    if ((uintptr_t)c.X % 16 || (uintptr_t)c.C % 16) {
        set_error("small-D variant needs 16-byte aligned X and C");
        return FTK_EALIGN;
    }
    const bool FT = c.ft != FTK_FT_OFF;
    SmallArgs a;
    a.X = (const float *)c.X;
    a.C = (const float *)c.C;
    a.hcn = (const float *)w.hcn;
    a.scal = w.scal;
    a.N = c.N;
    a.D = c.D;
    a.K = c.K;
    a.tpc = p.kch / 32;
    a.nch = p.nkc;
    a.tiles_total = (int)ceil_div(c.K, FT ? 30 : 32);
    a.nblocks = (int)p.workgroups;
    a.labels = c.labels;
    a.mindist = (float *)c.mindist;
    a.wl = w.wl;
    a.wl_count = w.wl_count;
    a.defer = c.ft == FTK_FT_STRICT ? 1 : 0;
    a.stats = c.stats;
    a.band_coef = p.band_coef;
    a.chk_v1 = (const float *)w.chk_v1;
    a.chk_v2 = (const float *)w.chk_v2;
    a.chk_s = (const float *)w.chk_s;
    a.faults = c.faults;
    a.n_faults = c.n_faults;
    a.ft_mode = (int)c.ft;
    a.ft_coef = p.ft_coef;
    a.widen = c.ft == FTK_FT_STRICT ? 1.0f : 0.0f;
    switch (p.D8 / 8) {
    case 1: launch_smalld_t<1>(a, p, FT, st); break;
    case 2: launch_smalld_t<2>(a, p, FT, st); break;
    case 3: launch_smalld_t<3>(a, p, FT, st); break;
    default: launch_smalld_t<4>(a, p, FT, st); break;
    }
    FTK_TRY_HIP(hipGetLastError());
    return FTK_OK;
}

}  // namespace ftk
