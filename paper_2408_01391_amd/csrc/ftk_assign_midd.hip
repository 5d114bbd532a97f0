// Mid-D assignment kernel (fp32, 32 < D <= 128, rows 16-byte aligned), with optional checksums.
//
// The register-resident blocking of the small-D kernel carried to rows of up to 128 features: a
// wave keeps the fragments of its 2 x 32 points (B operand) in registers for the whole sweep over
// K - up to 128 registers per lane - and the centroids (A operand) sit in LDS, all of them when
// K * D allows (256 centroids of 128 features fill a compute unit's LDS), else in chunks.  X is
// therefore read exactly once from memory, the sweep has no barrier and no global load in it, and
// the only vector work next to the matrix instructions is one 16-byte LDS read per eight of them
// plus the per-tile reduction.  (The generic kernel streams both operands through the D loop and
// keeps K-chunks of accumulators instead; it re-reads X once per chunk.)
//
// What differs from the small-D kernel is the end of a point: with D this large, re-evaluating a
// whole group of 16 rows exactly would cost a quarter of the sweep at K = 256.  Each lane instead
// keeps the 16 scores of its best tile (a conditional copy per tile: 16 selects per 128 matrix
// instructions) and takes the two best of them at the end; only centroids whose score lies inside
// the rounding bound of the best are evaluated in direct-difference form - the winner always (it
// also gives an accurate minimum distance), up to three more when they turn up - the two lanes of
// a point each covering the half of the features they hold.  More candidates than that, or a
// candidate in a tile that is not on record, send the point to the refine kernel.
//
// Fault tolerance (Sections 2.3, 4): tiles, checksum rows, verification, location and correction
// are those of the small-D kernel (30 centroids and two checksum rows per tile).  In strict mode
// the ambiguity band grows by the point's largest residual plus half the detection threshold; the
// ambiguous points are settled as above (there is no second sweep here).
#include <cmath>
#include <type_traits>

#include "ftk_internal.h"
#include "ftk_mma.h"
#include "ftk_smalld.h"

namespace ftk {

struct MidArgs {
    const float *X;
    const float *C;
    const float *hcn;    // half squared norms; beyond K: +inf (FT off) or unused (FT on)
    const double *scal;  // scal[0] = max_j ||c_j||^2
    int64_t N;
    int D, K;
    int tpc;          // tiles staged in LDS at a time
    int nch;          // chunks
    int tiles_total;  // ceil(K / centroids-per-tile)
    int nblocks;      // point blocks (waves * 64 points each)
    int32_t *labels;
    float *mindist;
    int32_t *wl;        // work-list of the refine kernel (point indices)
    int32_t *wl_count;  // [0] its length, [1] block counter
    ftk_ft_stats *stats;
    double band_coef;
    const float *chk_v1;  // [tiles_total*2][D8] plain checksum rows per (tile, lane group)
    const float *chk_v2;  // [tiles_total*2][D8] weighted (1..15) checksum rows
    const float *chk_s;   // [tiles_total*2][2]  matching sums of the half norms
    const ftk_fault *faults;
    int n_faults;
    int ft_mode;
    double ft_coef;  // detection threshold = ft_coef * (||x|| max||c|| + max||c||^2/2)
    float widen;     // 1 in strict mode, else 0
};

constexpr int MIDD_WAVES = 8;
constexpr int MIDD_PT = 2;

template <int NQ, bool FT>
__global__ __launch_bounds__(MIDD_WAVES * 64, 2) void assign_midd_kernel(MidArgs a)
{
    constexpr int THREADS = MIDD_WAVES * 64;
    constexpr int PT = MIDD_PT;
    using M = Mma<float>;
    using G = TileGeom<FT>;
    constexpr int SW = 8 * NQ + 4;   // LDS row stride in floats (16 bytes of padding)
    constexpr int TS = 32 * SW + 4;  // LDS tile stride
    constexpr int RG = G::RG;
    constexpr int D8 = 8 * NQ;
    extern __shared__ __align__(16) float lds[];
    float *ldsC = lds;                       // [tpc][TS]
    float *ldsH = lds + (size_t)a.tpc * TS;  // [tpc*32] accumulator start values, (tile, group, register) order
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
    int n_injected = 0, n_detected = 0, n_corrected = 0, n_recomputed = 0;
    float worst_resid = 0.f;

    for (int i = tid; i < SMALLD_LIST_CAP; i += THREADS) sh_wl[i] = -1;
    if (tid == 0) sh_wlcnt = 0;

    // stage tiles [ch*tpc, (ch+1)*tpc) into LDS: centroid rows (and checksum rows), zero-padded to
    // D8 features, plus the accumulator start values.  A thread keeps its 16-byte piece of the row
    // and walks the rows with a fixed stride; the loads are branch-free (clamped addresses, zeros
    // selected afterwards) and issued eight at a time, so a chunk costs two or three memory round
    // trips instead of one per row.
    // Threads t0 .. t0 + nthr - 1 of the workgroup take part.
    constexpr int PPR = 2 * NQ;  // 16-byte pieces per row
    auto stage_chunk = [&](int ch, int t0, int nthr) {
        const int rows = a.tpc * 32;
        const int ts = tid - t0;
        const int RSTEP = nthr / PPR;  // rows per pass
        const int st_pc = ts % PPR, st_r0 = ts / PPR;
        if (ts >= 0 && st_r0 < RSTEP) {
            for (int rb = st_r0; rb < rows; rb += 8 * RSTEP) {
                floatx4 f[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
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
                for (int u = 0; u < 8; ++u) {
                    const int rrow = rb + u * RSTEP;
                    if (rrow < rows)
                        *reinterpret_cast<floatx4 *>(ldsC + (size_t)(rrow >> 5) * TS + (rrow & 31) * SW + 4 * st_pc) = f[u];
                }
            }
        }
        for (int idx = ts; idx >= 0 && idx < rows; idx += nthr) {
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
    // With every tile resident the (only) chunk is staged inside the first unit of work, and the
    // two halves of the workgroup are set out of step on purpose: waves 0-3 request their points
    // first and wait while waves 4-7 stage the centroids and only then request theirs.  Each SIMD
    // holds one wave of either half, so from then on one of its two waves multiplies while the
    // other settles its points and fetches the next ones; started together, all waves of the chip
    // would fetch at the same moments and the matrix pipes would idle for the length of each burst.
    bool staged = false;


    // one unit of work of a wave: 64 points starting at p0, swept over all tiles and settled
    auto process = [&](int64_t p0, int blk) {
        floatx4 xf[PT][NQ];
        float xn[PT];
        float tau[PT];
        float inv_tau[PT];
        int force_refine[PT];
        float rmax[PT];
        TileBest best[PT];
        floatx16 bacc[PT];  // the scores of this lane's best tile
        auto request_points = [&]() {  // the loads only: nothing here waits for them
#pragma unroll
            for (int pt = 0; pt < PT; ++pt) {
                int64_t p = p0 + pt * 32 + col;
                if (p >= a.N) p = a.N - 1;
                const float *xrow = a.X + p * D;
#pragma unroll
                for (int q = 0; q < NQ; ++q) xf[pt][q] = load_frag<float, true>(xrow, 8 * q + 4 * g, D);
            }
        };
        auto start_points = [&]() {  // norms, thresholds, empty records
#pragma unroll
            for (int pt = 0; pt < PT; ++pt) {
                float s = 0.f;
#pragma unroll
                for (int q = 0; q < NQ; ++q)
#pragma unroll
                    for (int e = 0; e < 4; ++e) s = fmaf(xf[pt][q][e], xf[pt][q][e], s);
                xn[pt] = s + __shfl_xor(s, 32, 64);
                tau[pt] = (float)a.ft_coef * (sqrtf(xn[pt]) * cmax + 0.5f * cmax2);
                inv_tau[pt] = 1.0f / tau[pt];
                force_refine[pt] = 0;
                rmax[pt] = 0.f;
                best[pt].m1 = best[pt].m2 = M::neg_inf();
                best[pt].t1 = 0;
#pragma unroll
                for (int r = 0; r < 16; ++r) bacc[pt][r] = M::neg_inf();
            }
        };
        const bool head = resident && !staged && a.n_faults == 0;  // the out-of-step start (see above)
        const bool late = head && wave >= MIDD_WAVES / 2;
        if (!late) request_points();
        if (!head) start_points();

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

        // one output tile (local tile tl of the staged chunk, global tile T)
        auto compute_tile = [&](auto inj_tag, int tl, int T) {
            constexpr bool INJ = decltype(inj_tag)::value;
            floatx16 accs[PT];
            {
                const float *hp = ldsH + tl * 32 + g * 16;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const floatx4 h = *reinterpret_cast<const floatx4 *>(hp + 4 * i);
#pragma unroll
                    for (int pt = 0; pt < PT; ++pt) {
                        accs[pt][4 * i + 0] = h[0];
                        accs[pt][4 * i + 1] = h[1];
                        accs[pt][4 * i + 2] = h[2];
                        accs[pt][4 * i + 3] = h[3];
                    }
                }
            }
            const float *rowp = ldsC + (size_t)tl * TS + col * SW + 4 * g;
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                const floatx4 av = *reinterpret_cast<const floatx4 *>(rowp + 8 * q);
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int pt = 0; pt < PT; ++pt) accs[pt] = M::mma(av[e], xf[pt][q][e], accs[pt]);
            }
#pragma unroll
            for (int pt = 0; pt < PT; ++pt) {
                floatx16 acc = accs[pt];

                if constexpr (INJ) {  // fault injection (Section 2.1): flip one bit of one accumulator
                    for (int i = 0; i < nf; ++i) {
                        const ftk_fault f = sh_faults[i];
                        const int seq = (int)(f.tile % (unsigned)(a.tiles_total * PT));
                        if ((int)(f.wave % MIDD_WAVES) == wave && seq == T * PT + pt) {
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
                            // locate with the e2 = 1..15 weighted sum (Section 4.1); its reference is
                            // formed here on demand from the weighted checksum row
                            float s2 = 0.f;
#pragma unroll
                            for (int r = 0; r < RG; ++r) s2 = fmaf((float)(r + 1), acc[r], s2);
                            float ref2 = 0.f;
                            if (T < a.tiles_total) {
                                const float *v2 = a.chk_v2 + (size_t)(T * 2 + g) * D8;
                                float part = 0.f;  // this lane's half of the features
#pragma unroll
                                for (int q = 0; q < NQ; ++q) {
                                    const floatx4 vo = *reinterpret_cast<const floatx4 *>(v2 + 8 * q + 4 * g);
#pragma unroll
                                    for (int e = 0; e < 4; ++e) part = fmaf(xf[pt][q][e], vo[e], part);
                                }
                                // the other half: the partner lane's features against MY group's row
                                const float *v2p = a.chk_v2 + (size_t)(T * 2 + (1 - g)) * D8;
                                float cross = 0.f;  // my features against the partner group's row
#pragma unroll
                                for (int q = 0; q < NQ; ++q) {
                                    const floatx4 vp = *reinterpret_cast<const floatx4 *>(v2p + 8 * q + 4 * g);
#pragma unroll
                                    for (int e = 0; e < 4; ++e) cross = fmaf(xf[pt][q][e], vp[e], cross);
                                }
                                ref2 = part + __shfl_xor(cross, 32, 64) - a.chk_s[(T * 2 + g) * 2 + 1];
                            }
                            const float delta = resid;
                            const float fpos = (s2 - ref2) / delta;
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
                const bool c = tm > m1;
                best[pt].m2 = __builtin_amdgcn_fmed3f(m1, m2, tm);
                best[pt].t1 = c ? T : best[pt].t1;
                best[pt].m1 = max2f(m1, tm);
#pragma unroll
                for (int r = 0; r < RG; ++r) bacc[pt][r] = c ? acc[r] : bacc[pt][r];
            }
        };

        for (int ch = 0; ch < a.nch; ++ch) {
            if (head) {
                // nothing has read LDS yet: no barrier before; the one after also orders the
                // initialisation of the work-list buffer
                stage_chunk(ch, THREADS / 2, THREADS / 2);
                __syncthreads();
                staged = true;
                if (late) request_points();
                start_points();
            } else if (!resident || !staged) {
                __syncthreads();  // every wave is done with the previous chunk
                stage_chunk(ch, 0, THREADS);
                __syncthreads();
                staged = true;
            }
            const int tile0 = ch * a.tpc;
            const int ntile = min(a.tpc, a.tiles_total - tile0);
            if (nf > 0)
                for (int t = 0; t < ntile; ++t) compute_tile(std::true_type{}, t, tile0 + t);
            else
                for (int t = 0; t < ntile; ++t) compute_tile(std::false_type{}, t, tile0 + t);
        }

        // ---- settle each point: the lane's two best scores, the candidates inside the bound ----
#pragma unroll
        for (int pt = 0; pt < PT; ++pt) {
            if (FT) worst_resid = fmaxf(worst_resid, rmax[pt] * inv_tau[pt]);
            const int64_t p = p0 + pt * 32 + col;
            const bool live = p < a.N;
            // scores inside `bound` of each other cannot be ordered: rounding of the expanded form,
            // plus (strict FT) an undetected error below the detection threshold, which left its mark
            // in the residual of its tile: |error| <= |residual| + noise (taken as half the threshold)
            float bound = (float)a.band_coef * (sqrtf(xn[pt]) * cmax + 0.5f * cmax2);
            if (FT) bound += a.widen * (fmaxf(rmax[pt], __shfl_xor(rmax[pt], 32, 64)) + 0.5f * tau[pt]);
            const float v1 = best[pt].m1;  // the largest of the kept scores
            const float ov1 = __shfl_xor(v1, 32, 64);
            const float thr = fmaxf(v1, ov1) - bound;
            int r1 = 0, inside = 0;  // where it sits; how many of the kept scores lie inside the bound
#pragma unroll
            for (int r = RG - 1; r >= 0; --r) {
                r1 = bacc[pt][r] == v1 ? r : r1;
                inside += bacc[pt][r] >= thr ? 1 : 0;
            }
            // the second best of the kept scores is looked up only if some point of the wave has one
            // inside the bound
            float v2 = M::neg_inf();
            int r2 = 0;
            if (__any(inside >= 2)) {
#pragma unroll
                for (int r = 0; r < RG; ++r) {
                    const bool c2 = r != r1 && bacc[pt][r] > v2;
                    v2 = c2 ? bacc[pt][r] : v2;
                    r2 = c2 ? r : r2;
                }
            }
            // a third score of the best tile, or another tile's maximum: not on record
            const bool extra = inside >= 3 || best[pt].m2 >= thr;
            const bool mine_wins = v1 > ov1 || (v1 == ov1 && g == 0);
            const int j1 = G::centroid(best[pt].t1, g, r1), j2 = G::centroid(best[pt].t1, g, r2);
            const bool f1 = v1 >= thr, f2 = v2 >= thr;
            const int oj1 = __shfl_xor(j1, 32, 64), oj2 = __shfl_xor(j2, 32, 64);
            const bool of1 = __shfl_xor((int)f1, 32, 64) != 0, of2 = __shfl_xor((int)f2, 32, 64) != 0;
            const bool oextra = __shfl_xor((int)extra, 32, 64) != 0;
            const bool forced = (force_refine[pt] | __shfl_xor(force_refine[pt], 32, 64)) != 0;
            float dbest = __builtin_huge_valf();
            int jbest = 0x7fffffff;
            // direct-difference distance to centroid j: each lane of the pair sums the features it
            // holds, in feature order; the two halves are added (a commutative sum, so both lanes
            // get the same bits, and identical centroids the same distance)
            auto eval_row = [&](int j, bool take) {
                const bool real = take && j < a.K;
                const int jr = real ? j : 0;
                float d = 0.f;
                if (resident) {
                    const int T = jr / G::CPT, w = jr - T * G::CPT;
                    const int gg = FT ? w / 15 : (w >> 2) & 1;
                    const int r = FT ? w - 15 * gg : 0;
                    const int lr = FT ? (r >> 2) * 8 + gg * 4 + (r & 3) : w;
                    const float *c = ldsC + (size_t)T * TS + lr * SW + 4 * g;
#pragma unroll
                    for (int q = 0; q < NQ; ++q) {
                        const floatx4 cv = *reinterpret_cast<const floatx4 *>(c + 8 * q);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float t = xf[pt][q][e] - cv[e];
                            d = fmaf(t, t, d);
                        }
                    }
                } else {
                    const float *c = a.C + (size_t)jr * D;
#pragma unroll
                    for (int q = 0; q < NQ; ++q) {
                        const floatx4 cv = load_frag<float, true>(c, 8 * q + 4 * g, D);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float t = xf[pt][q][e] - cv[e];
                            d = fmaf(t, t, d);
                        }
                    }
                }
                d += __shfl_xor(d, 32, 64);
                const bool better = real & ((d < dbest) | ((d == dbest) & (j < jbest)));
                dbest = better ? d : dbest;
                jbest = better ? j : jbest;
            };
            // winner lane's best (always), then whatever else lies inside the bound
            eval_row(mine_wins ? j1 : oj1, true);
            const bool cb = mine_wins ? of1 : f1;  // the losing lane's best
            const bool cc = mine_wins ? f2 : of2;  // the winning lane's second
            const bool cd = mine_wins ? of2 : f2;  // the losing lane's second
            if (__any(cb)) eval_row(mine_wins ? oj1 : j1, cb);
            if (__any(cc)) eval_row(mine_wins ? j2 : oj2, cc);
            if (__any(cd)) eval_row(mine_wins ? oj2 : j2, cd);
            if (live && g == 0) {
                a.labels[p] = jbest == 0x7fffffff ? 0 : jbest;
                if (a.mindist) a.mindist[p] = dbest;
            }
            // NaN scores, more candidates than are on record, or a failed repair: exact recomputation
            const bool need = live && g == 0 && (!(thr == thr) || extra || oextra || forced);
            block_list_push(need, (int32_t)p, sh_wl, &sh_wlcnt, a.wl, a.wl_count);
        }
    };

    // Blocks of MIDD_WAVES units of 64 points.  With every tile resident and no faults listed the
    // waves are independent: each takes every gridDim-th block on its own, without barriers.
    // Otherwise the waves of a workgroup walk the blocks in step (chunks are staged, faults are
    // listed per block) and draw them from an atomic counter, one draw per block.
    int blk = blockIdx.x;
    while (blk < a.nblocks) {
        process(((int64_t)blk * MIDD_WAVES + wave) * (PT * 32), blk);
        if (resident && a.n_faults == 0) {
            blk += (int)gridDim.x;
            continue;
        }
        __syncthreads();
        if (tid == 0) sh_next = (int)gridDim.x + atomicAdd(a.wl_count + 1, 1);
        __syncthreads();
        blk = sh_next;
    }

    // hand the collected work-list entries over to the refine kernel
    __syncthreads();
    {
        const int n = min(sh_wlcnt, SMALLD_LIST_CAP);
        for (int i0 = 0; i0 < n; i0 += THREADS) {
            const int i = i0 + tid;
            const int32_t v = i < n ? sh_wl[i] : -1;
            worklist_push(v >= 0, v, a.wl, a.wl_count);
        }
    }

    // statistics: the number of comparisons is known in advance and added once; the other counters
    // are touched only when non-zero; the residual maximum is raised only by a wave that exceeds it
    if (a.stats && (FT || a.n_faults > 0)) {
        const int v[5] = {0, n_injected, n_detected, n_corrected, n_recomputed};
#pragma unroll
        for (int mask = 1; mask < 64; mask <<= 1) worst_resid = fmaxf(worst_resid, __shfl_xor(worst_resid, mask, 64));
        if (lane == 0) {
            unsigned long long *s = reinterpret_cast<unsigned long long *>(a.stats);
            if (FT && blockIdx.x == 0 && wave == 0)  // every (point, tile, lane group) is verified once
                atomicAdd(s, (unsigned long long)a.nblocks * MIDD_WAVES * PT * 64 * a.tiles_total);
            for (int i = 1; i < 5; ++i)
                if (v[i]) atomicAdd(s + i, (unsigned long long)v[i]);
            if (FT) {
                const unsigned long long mine = (unsigned long long)(fminf(worst_resid, 4000.f) * 1.0e6f);
                if (mine > *reinterpret_cast<volatile unsigned long long *>(s + 7)) atomicMax(s + 7, mine);
            }
        }
    }
}

bool midd_supported(ftk_dtype dtype, int D, int K)
{
    (void)K;
    return dtype == FTK_F32 && D > 32 && D <= 128 && D % 4 == 0;
}

// quads (8 features) of the compiled variant that holds D features
static int midd_nq(int D)
{
    const int nq = (int)ceil_div(D, 8);
    return nq <= 6 ? 6 : (nq <= 8 ? 8 : (nq <= 12 ? 12 : 16));
}

// Detection threshold coefficient: the form used for the small-D tiles (15 scores against one
// checksum, each a chain of D fused multiply-adds) with a safety factor for the longer chains:
// calibrated so that the largest fault-free residual seen stays below half the threshold (at
// D = 128 the residuals reach 0.55 of the unscaled form).
static constexpr double MIDD_FT_KAPPA = 1.6;
static double midd_ft_coef(int D)
{
    const double n = 15.0;
    return MIDD_FT_KAPPA * Mma<float>::kEps * n * (std::sqrt(n) + std::sqrt((double)D + 4.0));
}

void plan_midd(int64_t N, int D, int K, ftk_ft_mode ft, AssignPlan &p)
{
    const bool FT = ft != FTK_FT_OFF;
    p.variant = VAR_MIDD;
    p.TM = 32;
    p.TN = 32;
    p.D8 = 8 * midd_nq(D);  // rows are padded to the compiled width (checksum rows and LDS rows alike)
    p.PT = MIDD_PT;
    p.KT = 1;
    p.waves = MIDD_WAVES;
    const int SW = p.D8 + 4;
    const int tile_bytes = (32 * SW + 4) * 4 + 32 * 4;
    const int tiles_total = (int)ceil_div(K, FT ? 30 : 32);
    // one workgroup per compute unit: it can stage nearly all of the 160 KB (156 KB)
    int tpc = (156 * 1024) / tile_bytes;
    if (tpc > tiles_total) tpc = tiles_total;
    tpc = (int)ceil_div(tiles_total, ceil_div(tiles_total, tpc));  // equal chunks
    p.kch = tpc * 32;
    p.KC = tpc * 32;
    p.nkc = (int)ceil_div(tiles_total, tpc);
    p.DQ = p.D8 / 8;
    p.points_per_wg = p.waves * p.PT * 32;
    p.workgroups = ceil_div(N, p.points_per_wg);
    p.lds_bytes = (size_t)tpc * tile_bytes;
    p.grid = (int)(p.workgroups < 256 ? p.workgroups : 256);
    p.tiles_per_wave = tiles_total * p.PT;
    p.regs_per_tile = 16;
    p.hcn_pad_inf = !FT;
    p.ft_coef = midd_ft_coef(D);
    p.band_coef = 2.0 * (p.D8 + 4) * Mma<float>::kEps;
}

template <int NQ>
static void launch_midd_t(const MidArgs &a, const AssignPlan &p, bool ft, hipStream_t st)
{
    if (ft)
        hipLaunchKernelGGL((assign_midd_kernel<NQ, true>), dim3(p.grid), dim3(MIDD_WAVES * 64), p.lds_bytes, st, a);
    else
        hipLaunchKernelGGL((assign_midd_kernel<NQ, false>), dim3(p.grid), dim3(MIDD_WAVES * 64), p.lds_bytes, st, a);
}

ftk_status launch_assign_midd(const AssignCall &c, const AssignPlan &p, const Workspace &w, hipStream_t st)
{
    if ((uintptr_t)c.X % 16 || (uintptr_t)c.C % 16) {
        set_error("mid-D variant needs 16-byte aligned X and C");
        return FTK_EALIGN;
    }
    const bool FT = c.ft != FTK_FT_OFF;
    MidArgs a;
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
    case 6: launch_midd_t<6>(a, p, FT, st); break;
    case 8: launch_midd_t<8>(a, p, FT, st); break;
    case 12: launch_midd_t<12>(a, p, FT, st); break;
    default: launch_midd_t<16>(a, p, FT, st); break;
    }
    FTK_TRY_HIP(hipGetLastError());
    return FTK_OK;
}

}  // namespace ftk
