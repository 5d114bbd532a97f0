// Generic assignment kernel: any D, any K, fp32 and fp64.
//
// Computes, for every point, the centroid maximising the score
//     s_ij = x_i . c_j - ||c_j||^2 / 2  =  ( ||x_i||^2 - ||x_i - c_j||^2 ) / 2
// i.e. the expansion of Section 3.1.2 with the point norm (constant per point) left out of
// the comparison.  The contraction runs on the matrix cores; the accumulators start at
// -||c_j||^2/2 so the epilogue needs no norm arithmetic.  The arg-max is fused in registers
// (Sections 3.1.3-3.1.5): a workgroup owns a block of points and sweeps all K centroids, so
// no cross-workgroup combine (the lock/broadcast step of Section 3.1.4) is needed.
//
// Rounding: the expanded form cancels catastrophically when ||x||^2 dwarfs the gap between
// the two nearest centroids.  The epilogue therefore keeps the three best scores and the two
// best indices; a point whose runner-up lies within a rigorous rounding bound of the winner
// is settled by evaluating the two candidates in direct-difference form in double, and a
// point with three or more candidates inside the bound is queued for the refine kernel.
#include <cmath>
#include <type_traits>

#include "ftk_internal.h"
#include "ftk_mma.h"

namespace ftk {

template <typename T>
struct GenericArgs {
    const T *X;
    const T *C;
    const T *hcn;        // half squared norms, padded with zeros to nkc*KC entries
    const double *scal;  // scal[0] = max_j ||c_j||^2
    int64_t N;
    int D, K, D8, nkc;
    int32_t *labels;
    T *mindist;  // may be null
    int32_t *wl;
    int32_t *wl_count;
    int32_t *wg_refined;  // [gridDim.x] points this workgroup settled in place (read by the refine kernel)
    ftk_ft_stats *stats;
    double band_coef;  // ambiguity band = band_coef * (||x|| * max||c|| + max||c||^2 / 2)
    // fault tolerance / injection
    const T *chk_v1;   // [nkc][D8] per-chunk plain checksum row  (sum of the chunk's centroids)
    const T *chk_v2;   // [nkc][D8] per-chunk weighted checksum row (weights 1..KC)
    const double *chk_s;  // [nkc][2]  matching sums of the (rounded) half squared norms, in double
    const ftk_fault *faults;
    int n_faults;
    int ft_mode;
    double ft_coef;    // detection threshold = ft_coef * (||x|| * max||c|| + max||c||^2 / 2)
    double widen_coef; // half of it in strict mode (the ambiguity band grows by residual + noise), else 0
};

constexpr int GENERIC_MAX_FAULTS = 4;
#ifndef GENERIC_DQ_F32_KT4
#define GENERIC_DQ_F32_KT4 2
#endif

// Detection threshold = coefficient * u * B, B = ||x|| max||c|| + max||c||^2/2, for a check over
// n = KC scores of D features.  The coefficient models the rounding noise of a fault-free
// residual and carries a safety factor calibrated on the workloads and test shapes (largest
// fault-free residuals stay below a third of the threshold); a false alarm is harmless (the
// point is recomputed exactly), while a smaller threshold narrows the band of points that strict
// mode must settle exactly.
//   fp32: the reference and the score total are carried in double, so what is rounded in fp32 is
//     the n scores themselves (independent, each ~sqrt(D) u B), the tile sums of 16 scores, and
//     the quad-sized partial products of the reference against a checksum row of magnitude
//     n |c| (plus that row's own rounding):  sqrt(n) (sqrt(D+4) + 4) + 3 n / sqrt(D+4).
//   fp64: no wider type to carry the totals in; the running sums of n-fold magnitude dominate:
//     n (sqrt(n) + sqrt(D+4)).
template <typename T>
static double generic_ft_coef(int n, int D)
{
    const double dn = (double)n, dd = std::sqrt((double)D + 4.0);
    if (sizeof(T) == 4) return 1.7 * (std::sqrt(dn) * (dd + 4.0) + 3.0 * dn / dd);
    return 0.3 * dn * (std::sqrt(dn) + dd);
}

// Blocking per wave: PT = 2 point tiles by KT centroid tiles of accumulators (KT = 8: one point
// tile by eight centroid tiles, fp64 only), DQ quads per LDS
// stage, and the waves per SIMD the register budget is sized for.  KT = 4 is the workhorse (fp64
// tiles are 16x16, so it leaves room for a third resident wave).  For K of at most one or two
// tiles the stages hold little matrix work and the kernel is bound by the latency of the point
// loads; KT = 1 / 2 free the accumulator registers for more resident waves, i.e. more loads in
// flight.
// quads (8 features) per LDS stage.  Two everywhere: four for the fp32 workhorse (half as many
// barriers) needs 40 more registers for the point fragments, spills, and measured 8 % slower
// (c3: 170 against 158 us; with checksums 211 against 168 us).
constexpr int generic_dq(bool f32, int kt) { return (f32 && kt == 4) ? GENERIC_DQ_F32_KT4 : 2; }

template <typename T, int KT_>
struct GenericCfg {
    static constexpr int PT = KT_ == 8 ? 1 : 2, KT = KT_, WAVES = 4;
    static constexpr int DQ = generic_dq(sizeof(T) == 4, KT_);
    static constexpr int WAVES_PER_SIMD = KT_ == 8 ? 2 : (KT_ == 4 ? (sizeof(T) == 4 ? 2 : 3) : (KT_ == 2 ? 3 : 4));
};
// number of accumulator tiles used for a problem with K centroids
template <typename T>
constexpr int generic_kt(int K) { return K <= Mma<T>::TM ? 1 : (K <= 2 * Mma<T>::TM ? 2 : 4); }

// FULL: every stage holds real features only (D a multiple of the stage width) and every chunk
// real centroids only (K a multiple of the chunk) - the stage loop is then compiled without its
// per-quad, per-tile and per-element conditions: one straight run of matrix instructions per stage
// instead of a branch every KT of them, and no masking selects on the point fragments.
template <typename T, int KTV, bool ALIGNED, bool FT, bool FULL>
__global__ __launch_bounds__(256, (GenericCfg<T, KTV>::WAVES_PER_SIMD)) void assign_generic_kernel(GenericArgs<T> a)
{
    static_assert(ALIGNED || !FULL, "the condition-free stage loop is compiled for aligned rows only");
    using M = Mma<T>;
    using Cfg = GenericCfg<T, KTV>;
    using frag_t = typename M::frag_t;
    using acc_t = typename M::acc_t;
    constexpr int TM = M::TM, TN = M::TN, R = M::R, E = M::E;
    constexpr int PT = Cfg::PT, KT = Cfg::KT, KC = KT * TM;

    extern __shared__ __align__(16) unsigned char lds_raw[];
    __shared__ int sh_nf;
    __shared__ ftk_fault sh_faults[GENERIC_MAX_FAULTS];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int col = lane % TN;
    const int g = lane / TN;
    const int D = a.D;
    const int nq = a.D8 / 8;                        // quads in total

    const int64_t p0 = ((int64_t)blockIdx.x * Cfg::WAVES + wave) * (PT * TN);
    const T *xrow[PT];
#pragma unroll
    for (int pt = 0; pt < PT; ++pt) {
        int64_t p = p0 + pt * TN + col;
        if (p >= a.N) p = a.N - 1;  // clamped rows are computed and discarded
        xrow[pt] = a.X + p * D;
    }
    // FULL: the hot-loop loads address memory as a wave-uniform base plus a 32-bit lane offset
    // (one vector add per load instead of 64-bit pointer arithmetic): the rows of this workgroup
    // against its first row, the staged centroid pieces against C.  The launcher checks that the
    // offsets fit 32 bits.
    const char *const xbase = reinterpret_cast<const char *>(a.X + (int64_t)blockIdx.x * (Cfg::WAVES * PT * TN) * D);
    unsigned xoff[PT];
#pragma unroll
    for (int pt = 0; pt < PT; ++pt)
        xoff[pt] = (unsigned)((xrow[pt] - reinterpret_cast<const T *>(xbase)) + E * g) * (unsigned)sizeof(T);
    auto load_x = [&](int pt, int quad) -> frag_t {
        if constexpr (FULL)
            return *reinterpret_cast<const frag_t *>(xbase + (xoff[pt] + (unsigned)(quad * 8 * (int)sizeof(T))));
        else
            return load_frag_clamped<T, ALIGNED>(xrow[pt], quad * 8 + E * g, D);
    };

    // Epilogue state per point tile: best tile maximum, runner-up maximum over the OTHER tiles and
    // the best tile's number; the best tile's accumulators are parked in a per-lane LDS slot and the
    // arg-max inside it is taken once, at the end.  About one vector op per score for the maximum
    // instead of a full compare/select chain per score - fp32 matrix and vector work do not overlap
    // here - and the slot costs no registers.
    T bm1[PT], bm2[PT];
    int bt[PT];  // -1: no tile has produced a comparable score yet
    T xn[PT];
    T rmax[PT];             // largest checksum residual below the threshold over this point's chunks
    int force_refine[PT];   // a chunk of this point failed checksum correction (int, not bool:
                            // a bool array updated inside the rare branch lost its value when compiled)
#pragma unroll
    for (int pt = 0; pt < PT; ++pt) {
        bm1[pt] = bm2[pt] = M::neg_inf();
        bt[pt] = -1;
        xn[pt] = T(0);
        rmax[pt] = T(0);
        force_refine[pt] = 0;
    }
    const T cmax2 = (T)a.scal[0];
    const T cmax = sqrt(cmax2);
    // wave-uniform event counters (kept in scalar registers: counted with ballots)
    int n_injected = 0, n_detected = 0, n_corrected = 0, n_recomputed = 0;
    float worst_resid = 0.f;

    // faults aimed at this workgroup
    int nf = 0;
    if (a.n_faults > 0) {
        if (tid == 0) sh_nf = 0;
        __syncthreads();
        for (int i = tid; i < a.n_faults; i += 256) {
            if (a.faults[i].workgroup == blockIdx.x) {
                const int slot = atomicAdd(&sh_nf, 1);
                if (slot < GENERIC_MAX_FAULTS) sh_faults[slot] = a.faults[i];
            }
        }
        __syncthreads();
        nf = min(sh_nf, GENERIC_MAX_FAULTS);
    }

    // Centroid stages (DQ quads of one K-chunk, plus the chunk's checksum-row slice when FT is on)
    // go through two LDS buffers: the global loads of stage s+1 are issued before the matrix work
    // of stage s and land in LDS after it, so one barrier per stage is enough and the load latency
    // is covered by the matrix instructions.  The chunk's half-norms ride along with its first stage.
    constexpr int DQ = Cfg::DQ;
    constexpr int PPR = DQ * 8 / E;                      // 16-byte pieces per staged row
    constexpr int SB = DQ * 8 * (int)sizeof(T) + 16;     // row stride in bytes (bank spread)
    constexpr int STAGE_BYTES = (KC + 1) * SB;
    constexpr int NPIECES = KC * PPR;                    // 16-byte pieces per stage
    constexpr int NP = (NPIECES + 255) / 256;            // pieces per thread per stage
    static_assert(NPIECES % 256 == 0 || NPIECES < 256, "whole rounds over the workgroup, or a single partial one");
    static_assert(KC / E <= 64 && PPR <= 64, "extra pieces: half-norms on wave 0, checksum row on wave 1");
    unsigned char *const lds_hcn = lds_raw + 2 * STAGE_BYTES;
    // per-lane parking slots for the accumulators of the best tile so far ([pt][piece][thread])
    constexpr int BV = R / E;
    unsigned char *const lds_best = lds_hcn + 2 * KC * (int)sizeof(T);
    const int ndc = (nq + DQ - 1) / DQ;  // stages per K-chunk

    // Rows and pieces this thread stages are fixed; only the chunk and the feature offset move.
    int st_row[NP], st_pc[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        const int idx = min(tid + 256 * i, NPIECES - 1);  // surplus threads repeat the last piece (not stored)
        st_row[i] = idx / PPR;
        st_pc[i] = idx % PPR;
    }
    unsigned coff[NP];  // FULL: byte offset of this thread's pieces inside a chunk's first stage
#pragma unroll
    for (int i = 0; i < NP; ++i) coff[i] = (unsigned)(st_row[i] * D + st_pc[i] * E) * (unsigned)sizeof(T);
    const char *const cbase = reinterpret_cast<const char *>(a.C);
    frag_t pf[NP], pfx;
    // fetch only issues the loads (clamped into the matrix, so always valid); rows beyond K and
    // features beyond D are cleared when the stage is committed to LDS, i.e. after the matrix work
    // of the stage in between - a select right behind the load would make the wave wait for it here
    auto fetch = [&](int kc, int dc) {
        const int q0 = dc * DQ;
        const unsigned stage_off = (unsigned)(kc * KC * D + q0 * 8) * (unsigned)sizeof(T);  // wave-uniform
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            if constexpr (FULL) {
                pf[i] = *reinterpret_cast<const frag_t *>(cbase + (coff[i] + stage_off));
            } else {
                const int j = kc * KC + st_row[i];
                const int d0 = q0 * 8 + st_pc[i] * E;
                pf[i] = load_frag_clamped<T, ALIGNED>(a.C + (int64_t)min(j, a.K - 1) * D, d0, D);
            }
        }
#pragma unroll
        for (int e = 0; e < E; ++e) pfx[e] = T(0);
        if (dc == 0 && tid < KC / E)  // half-norms of the chunk (padded with zeros to nkc*KC entries)
            pfx = *reinterpret_cast<const frag_t *>(a.hcn + (size_t)kc * KC + tid * E);
        if (FT && tid >= 64 && tid < 64 + PPR && (q0 * 8 + (tid - 64) * E) < a.D8)
            pfx = *reinterpret_cast<const frag_t *>(a.chk_v1 + (size_t)kc * a.D8 + q0 * 8 + (tid - 64) * E);
    };
    auto commit = [&](int kc, int dc, int buf) {
        unsigned char *const base = lds_raw + buf * STAGE_BYTES;
        const int q0 = dc * DQ;
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const int idx = tid + 256 * i;
            if (NPIECES % 256 == 0 || idx < NPIECES) {
                const int j = kc * KC + st_row[i];
                const int d0 = q0 * 8 + st_pc[i] * E;
                *reinterpret_cast<frag_t *>(base + st_row[i] * SB + st_pc[i] * 16) =
                    FULL ? pf[i] : frag_keep<T>(pf[i], d0, D, j < a.K);
            }
        }
        if (dc == 0 && tid < KC / E) {  // stored negated: the accumulators start from -||c||^2/2
            frag_t neg;
#pragma unroll
            for (int e = 0; e < E; ++e) neg[e] = -pfx[e];
            *reinterpret_cast<frag_t *>(lds_hcn + ((kc & 1) * KC + tid * E) * (int)sizeof(T)) = neg;
        }
        if (FT && tid >= 64 && tid < 64 + PPR)
            *reinterpret_cast<frag_t *>(base + KC * SB + (tid - 64) * 16) = pfx;
    };

    // The point fragments of a whole stage (DQ quads) are fetched together, one stage ahead (the
    // prefetch wraps to stage 0 at the end of a K-chunk): the DQ pieces of a row are neighbours in
    // memory, and requesting them back to back consumes each cache line while it is resident
    // instead of coming back for its second half a thousand cycles later.
    // Features beyond D hold copies of valid ones: the staged centroid rows are zero there, so they
    // add nothing to the scores; the norm masks them explicitly.
    frag_t xs[PT][DQ];
#pragma unroll
    for (int pt = 0; pt < PT; ++pt)
#pragma unroll
        for (int q = 0; q < DQ; ++q) xs[pt][q] = load_x(pt, q);

    fetch(0, 0);
    commit(0, 0, 0);
    __syncthreads();
    int buf = 0;

    for (int kc = 0; kc < a.nkc; ++kc) {
        const int jbase = kc * KC;
        const int kt_act = min(KT, (a.K - jbase + TM - 1) / TM);  // tiles of this chunk with real centroids
        acc_t acc[PT][KT];
        {
            const T *const hl = reinterpret_cast<const T *>(lds_hcn) + (kc & 1) * KC;
#pragma unroll
            for (int t = 0; t < KT; ++t) {
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const T h = hl[t * TM + M::row(r, g)];
#pragma unroll
                    for (int pt = 0; pt < PT; ++pt) acc[pt][t][r] = h;
                }
            }
        }
        // x . (sum of the chunk's centroids), this lane's share of the features.  Each quad's four
        // products are summed in the working precision and added to a double: the rounding then
        // scales with one quad's partial sum, not with the running total of KC-fold magnitude.
        double ref1[PT];
#pragma unroll
        for (int pt = 0; pt < PT; ++pt) ref1[pt] = 0.0;

        for (int dc = 0; dc < ndc; ++dc) {
            const int q0 = dc * DQ;
            // next stage in sweep order (none after the last stage of the last chunk)
            const bool chunk_end = dc + 1 == ndc;
            const int kc_n = chunk_end ? kc + 1 : kc;
            const int dc_n = chunk_end ? 0 : dc + 1;
            const bool more = kc_n < a.nkc;
            if (more) fetch(kc_n, dc_n);
            const unsigned char *const sbuf = lds_raw + buf * STAGE_BYTES;
            frag_t xnx[PT][DQ];
            {
                const int qn0 = chunk_end ? 0 : q0 + DQ;
#pragma unroll
                for (int pt = 0; pt < PT; ++pt)
#pragma unroll
                    for (int q = 0; q < DQ; ++q)
                        xnx[pt][q] = load_x(pt, qn0 + q);
            }
#pragma unroll
            for (int q = 0; q < DQ; ++q) {
                if (FULL || q0 + q < nq) {
                    if (kc == 0) {
                        const int d0 = (q0 + q) * 8 + E * g;
#pragma unroll
                        for (int pt = 0; pt < PT; ++pt) {
                            const frag_t xm = FULL ? xs[pt][q] : frag_keep<T>(xs[pt][q], d0, D, true);
#pragma unroll
                            for (int e = 0; e < E; ++e) xn[pt] = fma(xm[e], xm[e], xn[pt]);
                        }
                    }
                    if (FT) {
                        // operand checksum on the vector ALU (Section 4.2): x . v1 over this lane's features
                        const frag_t v = *reinterpret_cast<const frag_t *>(
                            sbuf + KC * SB + q * (8 * (int)sizeof(T)) + g * 16);
#pragma unroll
                        for (int pt = 0; pt < PT; ++pt) {
                            T part = xs[pt][q][0] * v[0];
#pragma unroll
                            for (int e = 1; e < E; ++e) part = fma(xs[pt][q][e], v[e], part);
                            ref1[pt] += (double)part;
                        }
                    }
                    frag_t av[KT];
#pragma unroll
                    for (int t = 0; t < KT; ++t)
                        av[t] = *reinterpret_cast<const frag_t *>(
                            sbuf + (t * TM + lane % TM) * SB + q * (8 * (int)sizeof(T)) + g * 16);
                    // tiles that hold only padding rows (K small, or the last chunk) are skipped;
                    // their accumulators keep the start value of a zero row, exactly zero
#pragma unroll
                    for (int t = 0; t < KT; ++t) {
                        if (FULL || t < kt_act) {
#pragma unroll
                            for (int e = 0; e < E; ++e)
#pragma unroll
                                for (int pt = 0; pt < PT; ++pt)
                                    acc[pt][t] = M::mma(av[t][e], xs[pt][q][e], acc[pt][t]);
                        }
                    }
                }
            }
#pragma unroll
            for (int pt = 0; pt < PT; ++pt)
#pragma unroll
                for (int q = 0; q < DQ; ++q) xs[pt][q] = xnx[pt][q];
            if (more) commit(kc_n, dc_n, buf ^ 1);
            __syncthreads();
            buf ^= 1;
        }

        if (nf > 0) {  // fault injection (Section 2.1): flip one bit of one accumulator element
            using bits_t = typename std::conditional<sizeof(T) == 4, unsigned, unsigned long long>::type;
            for (int i = 0; i < nf; ++i) {
                const ftk_fault f = sh_faults[i];
                const int seq = (int)(f.tile % (unsigned)(a.nkc * PT * KT));
                if ((int)(f.wave % Cfg::WAVES) != wave || seq / (PT * KT) != kc) continue;
                const int fpt = (seq / KT) % PT, ft = seq % KT, fr = (int)(f.reg % R);
                const bool me = lane == (int)(f.lane & 63);
                const bits_t mask = (bits_t)1 << (f.bit % (8 * sizeof(T)));
#pragma unroll
                for (int pt = 0; pt < PT; ++pt)
#pragma unroll
                    for (int t = 0; t < KT; ++t)
#pragma unroll
                        for (int r = 0; r < R; ++r) {
                            bits_t b;
                            T v = acc[pt][t][r];
                            __builtin_memcpy(&b, &v, sizeof(T));
                            b ^= mask;
                            T flipped;
                            __builtin_memcpy(&flipped, &b, sizeof(T));
                            acc[pt][t][r] = (me && pt == fpt && t == ft && r == fr) ? flipped : v;
                        }
                n_injected += (int)__popcll(__ballot(me));
            }
        }

        if constexpr (FT) {
            // Verify the chunk before the arg-max reads it: for every point the KC scores must add
            // up to x . v1 - sum ||c||^2/2 (carried through the same feature loop).  A mismatch is
            // located with the weighted sum (weights 1..KC, Section 4.1) and corrected in place.
            const double s1ref = a.chk_s[2 * kc];
            // this lane's share of a point's KC scores: tile sums in the working precision, their
            // total in double (same reason as for the reference above)
            auto chunk_sum = [&](int pt) {
                double sd = 0.0;
#pragma unroll
                for (int t = 0; t < KT; ++t) {
                    T ts = acc[pt][t][0];
#pragma unroll
                    for (int r = 1; r < R; ++r) ts += acc[pt][t][r];
                    sd += (double)ts;
                }
                return sd;
            };
#pragma unroll
            for (int pt = 0; pt < PT; ++pt) {
                double s1d = chunk_sum(pt);
                double rfd = ref1[pt];
                T xnp = xn[pt];
#pragma unroll
                for (int mask = TN; mask < 64; mask <<= 1) {
                    s1d += shfl_xor_t(s1d, mask);
                    rfd += shfl_xor_t(rfd, mask);
                    xnp += shfl_xor_t(xnp, mask);
                }
                // xn is complete after the first chunk; later chunks reuse the same lanes' sums
                const T tau = (T)a.ft_coef * (sqrt(xnp) * cmax + (T)0.5 * cmax2);
                const T resid = (T)(s1d - (rfd - s1ref));
                const bool bad = !(fabs(resid) <= tau);
                if (__builtin_expect(__any(bad), 0)) {
                    n_detected += (int)__popcll(__ballot(bad && g == 0));
                    if (a.ft_mode >= FTK_FT_CORRECT) {
                        // weight of register (t, r) = its chunk row + 1 = wlane + (row at g = 0): the
                        // lane-dependent part is factored out so that the per-register weights are
                        // literals (as precomputed per-lane values they would sit in 64 registers
                        // for the whole kernel)
                        const double wlane = (double)(M::row(0, g) + 1);
                        double s2 = 0.0, s1l = 0.0;
#pragma unroll
                        for (int t = 0; t < KT; ++t)
#pragma unroll
                            for (int r = 0; r < R; ++r) {
                                s1l += (double)acc[pt][t][r];
                                s2 = fma((double)(t * TM + M::row(r, 0)), (double)acc[pt][t][r], s2);
                            }
                        s2 = fma(wlane, s1l, s2);
                        // weighted reference on demand: x . v2 over this lane's features
                        double r2 = 0.0;
                        for (int qq = 0; qq < nq; ++qq) {
                            const frag_t xv = load_frag<T, ALIGNED>(xrow[pt], qq * 8 + E * g, D);
                            const frag_t vv = *reinterpret_cast<const frag_t *>(a.chk_v2 + (size_t)kc * a.D8 + qq * 8 + E * g);
#pragma unroll
                            for (int e = 0; e < E; ++e) r2 = fma((double)xv[e], (double)vv[e], r2);
                        }
#pragma unroll
                        for (int mask = TN; mask < 64; mask <<= 1) {
                            s2 += shfl_xor_t(s2, mask);
                            r2 += shfl_xor_t(r2, mask);
                        }
                        r2 -= a.chk_s[2 * kc + 1];
                        const T fpos = (T)((s2 - r2) / (double)resid);
                        const T rpos = rint(fpos);
                        const bool finite = fabs(resid) < M::huge();
                        // the location is trusted only when the error stands far enough above the rounding
                        // noise of the weighted sum (weights up to KC) for the quotient to be accurate to a
                        // quarter; smaller detected errors are recomputed by the refine kernel instead
                        bool ok = bad && finite && fabs(resid) >= (T)(2 * KC) * tau && fabs(fpos - rpos) < (T)0.25 &&
                                  rpos >= (T)1 && rpos <= (T)KC;
                        const int wfix = ok ? (int)rpos - (M::row(0, g) + 1) : -1;  // relative to this lane's rows
#pragma unroll
                        for (int t = 0; t < KT; ++t)
#pragma unroll
                            for (int r = 0; r < R; ++r)
                                acc[pt][t][r] = (t * TM + M::row(r, 0) == wfix) ? acc[pt][t][r] - resid : acc[pt][t][r];
                        double s1b = chunk_sum(pt);
#pragma unroll
                        for (int mask = TN; mask < 64; mask <<= 1) s1b += shfl_xor_t(s1b, mask);
                        ok = ok && (fabs((T)(s1b - (rfd - s1ref))) <= tau);
                        n_corrected += (int)__popcll(__ballot(ok && g == 0));
                        n_recomputed += (int)__popcll(__ballot(bad && !ok && g == 0));
                        force_refine[pt] |= (bad && !ok) ? 1 : 0;
                    }
                }
                worst_resid = fmaxf(worst_resid, bad ? 0.f : (float)(fabs(resid) / tau));
                rmax[pt] = fmax(rmax[pt], bad ? T(0) : fabs(resid));
            }
        }

        // fused epilogue (rows beyond K only exist in the last chunk; the two variants keep the
        // common path free of the bounds select)
        auto epilogue = [&](auto tail_tag) {
            constexpr bool TAIL = decltype(tail_tag)::value;
#pragma unroll
            for (int pt = 0; pt < PT; ++pt) {
#pragma unroll
                for (int t = 0; t < KT; ++t) {
                    if (TAIL && t >= kt_act) continue;
                    if constexpr (TAIL) {
#pragma unroll
                        for (int r = 0; r < R; ++r)
                            acc[pt][t][r] = (jbase + t * TM + M::row(r, g) < a.K) ? acc[pt][t][r] : M::neg_inf();
                    }
                    T tm = acc[pt][t][0];
#pragma unroll
                    for (int r = 1; r < R; ++r) tm = fmax(tm, acc[pt][t][r]);
                    const T o1 = bm1[pt], o2 = bm2[pt];
                    const bool c = tm > o1;
                    bm2[pt] = M::med3(o1, o2, tm);
                    bm1[pt] = fmax(o1, tm);
                    bt[pt] = c ? kc * KT + t : bt[pt];
                    if (c) {  // rare after the first few tiles: park the tile in this lane's LDS slot
#pragma unroll
                        for (int i = 0; i < BV; ++i) {
                            frag_t w;
#pragma unroll
                            for (int e = 0; e < E; ++e) w[e] = acc[pt][t][i * E + e];
                            *reinterpret_cast<frag_t *>(lds_best + ((pt * BV + i) * 256 + tid) * 16) = w;
                        }
                    }
                }
            }
        };
        if (jbase + KC > a.K)
            epilogue(std::true_type{});
        else
            epilogue(std::false_type{});
    }

    // combine the lane groups that share a point
    uint64_t n_refined = 0;
#pragma unroll
    for (int pt = 0; pt < PT; ++pt) {
        // arg-max inside the saved best tile, then the runner-up of the other tiles as an
        // anonymous third entry (index -1: its centroid is not known)
        Top3<T> best;
        best.m1 = best.m2 = best.m3 = M::neg_inf();
        best.i1 = best.i2 = -1;
#pragma unroll
        for (int i = 0; i < BV; ++i) {
            const frag_t w = *reinterpret_cast<const frag_t *>(lds_best + ((pt * BV + i) * 256 + tid) * 16);
#pragma unroll
            for (int e = 0; e < E; ++e)
                best = top3_insert<T>(best, bt[pt] >= 0 ? w[e] : M::neg_inf(), bt[pt] * TM + M::row(i * E + e, g));
        }
        best = top3_insert<T>(best, bm2[pt], -1);
#pragma unroll
        for (int mask = TN; mask < 64; mask <<= 1) {
            const T b1 = shfl_xor_t(best.m1, mask), b2 = shfl_xor_t(best.m2, mask),
                    b3 = shfl_xor_t(best.m3, mask);
            const int j1 = shfl_xor_t(best.i1, mask), j2 = shfl_xor_t(best.i2, mask);
            best = top3_insert<T>(best, b1, j1);
            best = top3_insert<T>(best, b2, j2);
            best.m3 = M::med3(best.m2, best.m3, b3);  // b3 <= b2 can never pass m2
            xn[pt] += shfl_xor_t(xn[pt], mask);
        }
        const T m1 = best.m1, m2 = best.m2, m3 = best.m3;
        const int i1 = best.i1 < 0 ? 0 : best.i1, i2 = best.i2;
        // After the exchange both partners hold the same multiset of values but may order
        // equal scores differently; everything below only depends on values, and candidate
        // indices are made symmetric by ordering the pair.
        const int64_t p = p0 + pt * TN + col;
        const bool live = p < a.N;
        // scores inside `bound` of each other cannot be ordered: rounding of the expanded form,
        // plus (strict FT) an undetected error below the detection threshold
        // (strict FT: an error that stayed below the detection threshold shows in the residual of
        // its chunk, |error| <= |residual| + rounding noise, the noise taken as at most half the
        // threshold; widen_coef is half the threshold coefficient in strict mode, else zero)
        T bound = (T)(a.band_coef + (FT ? a.widen_coef : 0.0)) * (sqrt(xn[pt]) * cmax + (T)0.5 * cmax2);
        if (FT && a.widen_coef > 0.0) bound += rmax[pt];
        const bool amb2 = (m1 - m2) <= bound;
        // a runner-up whose centroid is unknown cannot be settled in place: leave it to the refine kernel
        const bool amb3 = ((m1 - m3) <= bound) || force_refine[pt] != 0 || (amb2 && i2 < 0);
        int label = i1;
        T dist = xn[pt] - (T)2 * m1;
        dist = dist > T(0) ? dist : T(0);
        worklist_push(live && amb3 && g == 0, (int32_t)p, a.wl, a.wl_count);
        if (live && amb3) {
            // three or more candidates: settled by the refine kernel
        } else if (live && amb2) {
            // two candidates: lane groups 0/1 each evaluate one of them exactly
            const int ja = min(i1, i2), jb = max(i1, i2);
            const int mine = (g & 1) ? jb : ja;
            const double dm = exact_sqdist<T, ALIGNED>(xrow[pt], a.C + (int64_t)mine * D, D);
            const double dother = shfl_xor_t(dm, TN);
            const double da = (g & 1) ? dother : dm;
            const double db = (g & 1) ? dm : dother;
            label = (db < da) ? jb : ja;  // equal distances: lower index
            dist = (T)((db < da) ? db : da);
            if (g == 0) n_refined += 1;
        }
        if (live && g == 0) {
            a.labels[p] = label;
            if (a.mindist) a.mindist[p] = dist;
        }
    }
    // Statistics.  Several thousand waves adding to the same few words would keep the memory
    // system busy long after the last wave has ended, so: the number of comparisons made is known
    // in advance and added once; the other counters are touched only when non-zero (i.e. when a
    // fault was seen); the residual maximum is read first and raised only by a wave that exceeds it.
    if (a.stats && (FT || a.n_faults > 0)) {
        const int v[5] = {0, n_injected, n_detected, n_corrected, n_recomputed};
#pragma unroll
        for (int mask = 1; mask < 64; mask <<= 1) worst_resid = fmaxf(worst_resid, __shfl_xor(worst_resid, mask, 64));
        if (lane == 0) {
            unsigned long long *sp = reinterpret_cast<unsigned long long *>(a.stats);
            if (FT && blockIdx.x == 0 && wave == 0)
                atomicAdd(sp, (unsigned long long)gridDim.x * Cfg::WAVES * PT * TN * a.nkc);
            for (int i = 1; i < 5; ++i)
                if (v[i]) atomicAdd(sp + i, (unsigned long long)v[i]);
            if (FT) {
                const unsigned long long mine = (unsigned long long)(fminf(worst_resid, 4000.f) * 1.0e6f);
                if (mine > *reinterpret_cast<volatile unsigned long long *>(sp + 7)) atomicMax(sp + 7, mine);
            }
        }
    }
    if (a.stats) {
        // points settled in place: one plain store per workgroup, summed by the refine kernel
        // (an atomic per wave on the one counter kept the dispatch open for tens of microseconds)
        __shared__ int sh_refined;
        int n = (int)n_refined;
#pragma unroll
        for (int mask = 1; mask < 64; mask <<= 1) n += __shfl_xor(n, mask, 64);
        if (tid == 0) sh_refined = 0;
        __syncthreads();
        if (lane == 0 && n) atomicAdd(&sh_refined, n);
        __syncthreads();
        if (tid == 0) a.wg_refined[blockIdx.x] = sh_refined;
    }
}

// The end of a batch: every thread holds its best (distance, index) per point; combined over the
// wave, then over the four waves, lowest index on equal distances; written by one thread per point.
template <typename T, int P>
__device__ __forceinline__ void refine_settle(double (&best)[P], int (&bj)[P], const int32_t *__restrict__ wl, int first,
                                              int np, int32_t *labels, T *mindist, double (*sh_best)[8], int (*sh_j)[8])
{
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
#pragma unroll
    for (int u = 0; u < P; ++u) {
#pragma unroll
        for (int mask = 1; mask < 64; mask <<= 1) {
            const double ob = __shfl_xor(best[u], mask, 64);
            const int oj = __shfl_xor(bj[u], mask, 64);
            const bool take = ob < best[u] || (ob == best[u] && oj < bj[u]);
            best[u] = take ? ob : best[u];
            bj[u] = take ? oj : bj[u];
        }
        if (lane == 0) {
            sh_best[wave][u] = best[u];
            sh_j[wave][u] = bj[u];
        }
    }
    __syncthreads();
    if (tid < np) {
        double b = sh_best[0][tid];
        int j = sh_j[0][tid];
#pragma unroll
        for (int v = 1; v < 4; ++v) {
            const double ob = sh_best[v][tid];
            const int oj = sh_j[v][tid];
            if (ob < b || (ob == b && oj < j)) {
                b = ob;
                j = oj;
            }
        }
        const int64_t p = wl[first + tid];
        labels[p] = j == 0x7fffffff ? 0 : j;
        if (mindist) mindist[p] = (T)b;
    }
    __syncthreads();  // the slots are rewritten for the next batch
}

// Exact settlement of the queued points: all K distances of a point in the direct-difference form
// (double), then the arg-min with the lowest index on ties.  A workgroup settles a batch of up to
// P queued points at a time: thread t owns centroid rows t, t + 256, ... and evaluates each of
// them against all points of the batch, so a centroid row is fetched once per batch instead of
// once per point (with thousands of queued points the kernel was bound by re-reading C from L2:
// K*D bytes per point).  The batch size adapts to the queue: one point per workgroup while the
// queue is shorter than the grid (the work is then a chain of memory latencies and is spread as
// widely as possible), up to P = 8 beyond.  Point rows are read with wave-uniform addresses (one
// cache line broadcast per load).  Every (point, centroid) sum adds the features in index order
// into one accumulator, so identical centroids tie exactly whatever the batch size.
template <typename T, bool ALIGNED, int JU, int P>
__device__ __forceinline__ void refine_batch(const T *__restrict__ X, const T *__restrict__ C, int D, int K,
                                             const int32_t *__restrict__ wl, int first, int np,
                                             int32_t *labels, T *mindist, double (*sh_best)[8], int (*sh_j)[8])
{
    constexpr int E = Mma<T>::E;
    // about sixteen 16-byte loads in flight per thread (centroid rows and point rows together)
    constexpr int DU_RAW = 16 / (JU + P - 1);
    constexpr int DU = DU_RAW >= 16 ? 16 : (DU_RAW >= 8 ? 8 : (DU_RAW >= 4 ? 4 : (DU_RAW >= 2 ? 2 : 1)));
    using F = typename Mma<T>::frag_t;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const T *x[P];
    int64_t pidx[P];
#pragma unroll
    for (int u = 0; u < P; ++u) {  // slots beyond the batch repeat its last point
        pidx[u] = wl[first + min(u, np - 1)];
        x[u] = X + pidx[u] * D;
    }
    double best[P];
    int bj[P];
#pragma unroll
    for (int u = 0; u < P; ++u) {
        best[u] = __builtin_huge_val();
        bj[u] = 0x7fffffff;
    }
    for (int j0 = tid; j0 < K; j0 += 256 * JU) {
        const T *c[JU];
        double s[JU][P];
#pragma unroll
        for (int r = 0; r < JU; ++r) {
            c[r] = C + (int64_t)min(j0 + 256 * r, K - 1) * D;
#pragma unroll
            for (int u = 0; u < P; ++u) s[r][u] = 0.0;
        }
        for (int d0 = 0; d0 < D; d0 += E * DU) {
            F cf[JU][DU], xf[P][DU];
#pragma unroll
            for (int r = 0; r < JU; ++r)
#pragma unroll
                for (int v = 0; v < DU; ++v) cf[r][v] = load_frag_clamped<T, ALIGNED>(c[r], d0 + v * E, D);
#pragma unroll
            for (int u = 0; u < P; ++u)
#pragma unroll
                for (int v = 0; v < DU; ++v) xf[u][v] = load_frag_clamped<T, ALIGNED>(x[u], d0 + v * E, D);
#pragma unroll
            for (int v = 0; v < DU; ++v) {
                // aligned rows hold whole fragments: a fragment is inside the row or (clamped copy)
                // skipped as a whole, a wave-uniform decision; otherwise elements are masked one by one
                if (ALIGNED && d0 + v * E >= D) continue;
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    const bool keep = ALIGNED || d0 + v * E + e < D;
                    double cd[JU];
#pragma unroll
                    for (int r = 0; r < JU; ++r) cd[r] = (double)cf[r][v][e];
#pragma unroll
                    for (int u = 0; u < P; ++u) {
                        const double xd = (double)xf[u][v][e];
#pragma unroll
                        for (int r = 0; r < JU; ++r) {
                            const double diff = keep ? xd - cd[r] : 0.0;
                            s[r][u] = fma(diff, diff, s[r][u]);
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int r = 0; r < JU; ++r) {  // j increases within a thread: first minimum kept
            const int j = j0 + 256 * r;
#pragma unroll
            for (int u = 0; u < P; ++u) {
                const bool better = j < K && s[r][u] < best[u];
                best[u] = better ? s[r][u] : best[u];
                bj[u] = better ? j : bj[u];
            }
        }
    }
    refine_settle<T, P>(best, bj, wl, first, np, labels, mindist, sh_best, sh_j);
}

// The same for aligned rows of 16 fragments and more: L lanes share a centroid row (8, or the whole
// wave from 128 fragments on), each taking every L-th 16-byte fragment.  With a thread per row a
// load instruction touches 64 different rows - 64 requests to the vector cache, a whole line read
// for each 16 bytes used - and the kernel's time was those requests (2^18 x 128, K = 256: 12 us
// for a few hundred points); here an instruction reads runs of 128 bytes and more.  The L partial
// sums of a row are added by the same tree for every row, so identical centroids still tie exactly.
template <typename T, int L, int P>
__device__ __forceinline__ void refine_batch_wide(const T *__restrict__ X, const T *__restrict__ C, int D, int K,
                                                  const int32_t *__restrict__ wl, int first, int np,
                                                  int32_t *labels, T *mindist, double (*sh_best)[8], int (*sh_j)[8])
{
    constexpr int E = Mma<T>::E;
    constexpr int ROWS = 256 / L;          // centroid rows per pass of the workgroup
    constexpr int JU = P >= 4 ? 2 : 4;     // rows in flight per thread
    constexpr int DU = P >= 4 ? 2 : 4;     // fragments per row in flight
    using F = typename Mma<T>::frag_t;
    const int tid = threadIdx.x;
    const int sub = tid & (L - 1);
    const int slot = tid / L;
    const int nfrag = D / E;
    const T *x[P];
#pragma unroll
    for (int u = 0; u < P; ++u)  // slots beyond the batch repeat its last point
        x[u] = X + (int64_t)wl[first + min(u, np - 1)] * D;
    double best[P];
    int bj[P];
#pragma unroll
    for (int u = 0; u < P; ++u) {
        best[u] = __builtin_huge_val();
        bj[u] = 0x7fffffff;
    }
    for (int j0 = slot; j0 < K; j0 += ROWS * JU) {
        const T *c[JU];
        double s[JU][P];
#pragma unroll
        for (int r = 0; r < JU; ++r) {
            c[r] = C + (int64_t)min(j0 + ROWS * r, K - 1) * D;
#pragma unroll
            for (int u = 0; u < P; ++u) s[r][u] = 0.0;
        }
        for (int f0 = sub; f0 < nfrag; f0 += L * DU) {
            F cf[JU][DU], xf[P][DU];
#pragma unroll
            for (int v = 0; v < DU; ++v) {
                const int off = min(f0 + L * v, nfrag - 1) * E;
#pragma unroll
                for (int r = 0; r < JU; ++r) cf[r][v] = *reinterpret_cast<const F *>(c[r] + off);
#pragma unroll
                for (int u = 0; u < P; ++u) xf[u][v] = *reinterpret_cast<const F *>(x[u] + off);
            }
#pragma unroll
            for (int v = 0; v < DU; ++v) {
                const bool keep = f0 + L * v < nfrag;  // a clamped copy beyond the row counts nothing
#pragma unroll
                for (int e = 0; e < E; ++e) {
#pragma unroll
                    for (int u = 0; u < P; ++u) {
                        const double xd = (double)xf[u][v][e];
#pragma unroll
                        for (int r = 0; r < JU; ++r) {
                            const double diff = keep ? xd - (double)cf[r][v][e] : 0.0;
                            s[r][u] = fma(diff, diff, s[r][u]);
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int r = 0; r < JU; ++r) {  // j increases within a thread: first minimum kept
            const int j = j0 + ROWS * r;
#pragma unroll
            for (int u = 0; u < P; ++u) {
                double t = s[r][u];
#pragma unroll
                for (int mask = L >> 1; mask >= 1; mask >>= 1) t += __shfl_xor(t, mask, 64);
                const bool better = j < K && t < best[u];
                best[u] = better ? t : best[u];
                bj[u] = better ? j : bj[u];
            }
        }
    }
    refine_settle<T, P>(best, bj, wl, first, np, labels, mindist, sh_best, sh_j);
}

template <typename T, bool ALIGNED, int JU, int L>
__global__ __launch_bounds__(256) void refine_kernel(const T *__restrict__ X, const T *__restrict__ C, int D, int K,
                                                     const int32_t *__restrict__ wl, const int32_t *__restrict__ wl_count,
                                                     int32_t *labels, T *mindist, ftk_ft_stats *stats,
                                                     const int32_t *__restrict__ wg_refined, int n_wg)
{
    __shared__ double sh_best[4][8];
    __shared__ int sh_j[4][8];
    const int count = *wl_count;
    // batch size: the smallest power of two that lets the grid cover the queue in one round, at most 8
    const int per_wg = (count + (int)gridDim.x - 1) / (int)gridDim.x;
    const int bs = per_wg <= 1 ? 1 : (per_wg <= 2 ? 2 : (per_wg <= 4 ? 4 : 8));
    const int nbatch = (count + bs - 1) / bs;
    for (int b = blockIdx.x; b < nbatch; b += gridDim.x) {
        const int first = b * bs;
        const int np = min(bs, count - first);
        if constexpr (L > 1) {
            if (bs == 1)
                refine_batch_wide<T, L, 1>(X, C, D, K, wl, first, np, labels, mindist, sh_best, sh_j);
            else if (bs == 2)
                refine_batch_wide<T, L, 2>(X, C, D, K, wl, first, np, labels, mindist, sh_best, sh_j);
            else if (bs == 4)
                refine_batch_wide<T, L, 4>(X, C, D, K, wl, first, np, labels, mindist, sh_best, sh_j);
            else
                refine_batch_wide<T, L, 8>(X, C, D, K, wl, first, np, labels, mindist, sh_best, sh_j);
        } else {
            if (bs == 1)
                refine_batch<T, ALIGNED, JU, 1>(X, C, D, K, wl, first, np, labels, mindist, sh_best, sh_j);
            else if (bs == 2)
                refine_batch<T, ALIGNED, (JU > 4 ? 4 : JU), 2>(X, C, D, K, wl, first, np, labels, mindist, sh_best, sh_j);
            else if (bs == 4)
                refine_batch<T, ALIGNED, (JU > 2 ? 2 : JU), 4>(X, C, D, K, wl, first, np, labels, mindist, sh_best, sh_j);
            else
                refine_batch<T, ALIGNED, (JU > 2 ? 2 : JU), 8>(X, C, D, K, wl, first, np, labels, mindist, sh_best, sh_j);
        }
    }
    if (stats && blockIdx.x == 0) {
        // statistics: queued points plus those the main kernel's workgroups settled in place
        __shared__ int sh_total;
        if (threadIdx.x == 0) sh_total = count;
        __syncthreads();
        int n = 0;
        for (int i = threadIdx.x; i < n_wg; i += 256) n += wg_refined[i];
#pragma unroll
        for (int mask = 1; mask < 64; mask <<= 1) n += __shfl_xor(n, mask, 64);
        if ((threadIdx.x & 63) == 0 && n) atomicAdd(&sh_total, n);
        __syncthreads();
        if (threadIdx.x == 0 && sh_total > 0)
            atomicAdd((unsigned long long *)&stats->refined, (unsigned long long)sh_total);
    }
}

template <typename T>
static ftk_status launch_generic_t(const AssignCall &c, const AssignPlan &p, const Workspace &w,
                                   hipStream_t st)
{
    GenericArgs<T> a;
    a.X = (const T *)c.X;
    a.C = (const T *)c.C;
    a.hcn = (const T *)w.hcn;
    a.scal = w.scal;
    a.N = c.N;
    a.D = c.D;
    a.K = c.K;
    a.D8 = p.D8;
    a.nkc = p.nkc;
    a.labels = c.labels;
    a.mindist = (T *)c.mindist;
    a.wl = w.wl;
    a.wl_count = w.wl_count;
    a.wg_refined = w.wg_refined;
    a.stats = c.stats;
    // Rounding bound of one score (band_coef, set by plan_generic).  On this hardware the matrix instructions (fp32 and fp64) return
    // exactly the chain of fused multiply-adds over the contraction index in order, each rounded to
    // nearest even (checked against fmaf/fma chains on several hundred thousand random operands).
    // A score is therefore a chain of D8 fused steps started from the rounded -||c||^2/2; every
    // step errs by at most u times its partial sum, and the partial sums stay below
    // B = |x|.|c| + ||c||^2/2 (up to 1 + D8 u), so |fl(s) - s| <= (D8 + 1) u B (1 + D8 u).
    // Two scores are compared: twice that, with D8 + 4 absorbing the second-order factor and the
    // fp32 evaluation of B itself.
    a.band_coef = p.band_coef;
    a.chk_v1 = (const T *)w.chk_v1;
    a.chk_v2 = (const T *)w.chk_v2;
    a.chk_s = w.chk_sd;
    a.faults = c.faults;
    a.n_faults = c.n_faults;
    a.ft_mode = (int)c.ft;
    a.ft_coef = p.ft_coef;
    a.widen_coef = c.ft == FTK_FT_STRICT ? 0.5 * a.ft_coef : 0.0;
    const bool aligned = (c.D % Mma<T>::E == 0) && ((uintptr_t)c.X % 16 == 0) && ((uintptr_t)c.C % 16 == 0);
    const bool ft = c.ft != FTK_FT_OFF;
    dim3 grid((unsigned)p.workgroups), block(256);
    // whole stages and whole chunks: the condition-free stage loop
    // (and 32-bit byte offsets inside C and inside a workgroup's block of rows)
    const bool full = aligned && c.D % (8 * p.DQ) == 0 && c.K % p.KC == 0 &&
                      (double)c.K * c.D * sizeof(T) < 4.0e9 && (double)p.points_per_wg * c.D * sizeof(T) < 4.0e9;
#define FTK_LAUNCH_GEN(KV, AL, F, FU) \
    hipLaunchKernelGGL((assign_generic_kernel<T, KV, AL, F, FU>), grid, block, p.lds_bytes, st, a)
#define FTK_LAUNCH_GEN_K(KV)                          \
    do {                                              \
        if (full && ft) FTK_LAUNCH_GEN(KV, true, true, true);          \
        else if (full) FTK_LAUNCH_GEN(KV, true, false, true);          \
        else if (aligned && ft) FTK_LAUNCH_GEN(KV, true, true, false); \
        else if (aligned) FTK_LAUNCH_GEN(KV, true, false, false);      \
        else if (ft) FTK_LAUNCH_GEN(KV, false, true, false);           \
        else FTK_LAUNCH_GEN(KV, false, false, false);                  \
    } while (0)
    if (p.KT == 8) FTK_LAUNCH_GEN_K(8);
    else if (p.KT == 4) FTK_LAUNCH_GEN_K(4);
    else if (p.KT == 2) FTK_LAUNCH_GEN_K(2);
    else FTK_LAUNCH_GEN_K(1);
#undef FTK_LAUNCH_GEN_K
#undef FTK_LAUNCH_GEN
    FTK_TRY_HIP(hipGetLastError());
    return FTK_OK;
}

ftk_status launch_assign_generic(const AssignCall &c, const AssignPlan &p, const Workspace &w,
                                 hipStream_t st)
{
    return c.dtype == FTK_F32 ? launch_generic_t<float>(c, p, w, st)
                              : launch_generic_t<double>(c, p, w, st);
}

template <typename T>
static void launch_refine_t(const AssignCall &c, const Workspace &w, int n_wg, hipStream_t st)
{
    const bool aligned = (c.D % Mma<T>::E == 0) && ((uintptr_t)c.X % 16 == 0) && ((uintptr_t)c.C % 16 == 0);
    dim3 grid(1024), block(256);
#define FTK_LAUNCH_REFINE(AL, JU, LV)                                                                      \
    hipLaunchKernelGGL((refine_kernel<T, AL, JU, LV>), grid, block, 0, st, (const T *)c.X, (const T *)c.C, \
                       c.D, c.K, w.wl, w.wl_count, c.labels, (T *)c.mindist, c.stats, w.wg_refined, n_wg)
#define FTK_LAUNCH_REFINE_J(JU)                   \
    do {                                          \
        if (aligned) FTK_LAUNCH_REFINE(true, JU, 1); \
        else FTK_LAUNCH_REFINE(false, JU, 1);        \
    } while (0)
    // sixteen 16-byte loads in flight per thread: short rows leave room for more rows at once
    const int nfrag = (int)ceil_div(c.D, Mma<T>::E);
    // long aligned rows: lanes share a row (see refine_batch_wide)
    if (aligned && nfrag >= 128) FTK_LAUNCH_REFINE(true, 1, 64);
    else if (aligned && nfrag >= 16) FTK_LAUNCH_REFINE(true, 1, 8);
    else if (nfrag <= 2) FTK_LAUNCH_REFINE_J(8);
    else if (nfrag <= 4) FTK_LAUNCH_REFINE_J(4);
    else if (nfrag <= 8) FTK_LAUNCH_REFINE_J(2);
    else FTK_LAUNCH_REFINE_J(1);
#undef FTK_LAUNCH_REFINE_J
#undef FTK_LAUNCH_REFINE
}

ftk_status launch_refine(const AssignCall &c, const Workspace &w, int n_wg, hipStream_t st)
{
    if (c.dtype == FTK_F32)
        launch_refine_t<float>(c, w, n_wg, st);
    else
        launch_refine_t<double>(c, w, n_wg, st);
    FTK_TRY_HIP(hipGetLastError());
    return FTK_OK;
}

void plan_generic(ftk_dtype dtype, int64_t N, int D, int K, AssignPlan &p)
{
    const bool f32 = dtype == FTK_F32;
    p.variant = VAR_GENERIC;
    p.TM = f32 ? Mma<float>::TM : Mma<double>::TM;
    p.TN = f32 ? Mma<float>::TN : Mma<double>::TN;
    p.KT = f32 ? generic_kt<float>(K) : generic_kt<double>(K);
    // fp64, long rows, more than one chunk of centroids: eight tiles of ONE point tile per wave sweep
    // twice as many centroids per pass over X, which is what these shapes wait for (X is re-read
    // once per chunk and 16x16 tiles make chunks small); measured 3-14 % faster from D = 512 on,
    // slower below (the point fragments are reused half as often).  fp32 tiles are 32 wide and
    // the same layout measured slower there.
    if (!f32 && D >= 512 && K > 4 * Mma<double>::TM) p.KT = 8;
    if (g_tuning.kt > 0) p.KT = g_tuning.kt;
    p.PT = p.KT == 8 ? 1 : 2;
    p.waves = 4;
    p.KC = p.KT * p.TM;
    p.nkc = (int)ceil_div(K, p.KC);
    p.D8 = (int)ceil_div(D, 8) * 8;
    p.DQ = generic_dq(f32, p.KT);
    p.points_per_wg = p.waves * p.PT * p.TN;
    p.workgroups = ceil_div(N, p.points_per_wg);
    p.tiles_per_wave = p.nkc * p.PT * p.KT;
    p.regs_per_tile = f32 ? Mma<float>::R : Mma<double>::R;
    const size_t esz = f32 ? 4 : 8;
    // two stage buffers of KC+1 rows, two half-norm buffers, the best-tile slots of 256 lanes
    p.lds_bytes = 2 * (size_t)(p.KC + 1) * (8 * p.DQ * esz + 16) + 2 * (size_t)p.KC * esz +
                  (size_t)p.PT * p.regs_per_tile * esz * 256;
    p.hcn_pad_inf = false;
    p.grid = (int)p.workgroups;
    p.kch = p.KC;
    p.ft_coef = f32 ? generic_ft_coef<float>(p.KC, D) * Mma<float>::kEps
                    : generic_ft_coef<double>(p.KC, D) * Mma<double>::kEps;
    p.band_coef = 2.0 * (p.D8 + 4) * (f32 ? Mma<float>::kEps : Mma<double>::kEps);
}

}  // namespace ftk
