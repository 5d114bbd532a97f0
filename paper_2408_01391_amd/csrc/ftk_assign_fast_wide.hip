// Fast assignment for fp32 data with 32 < D <= 128: the contraction on the bf16 matrix
// instructions with both operands split into two bf16 pieces, in the register-resident blocking
// of the fp32 mid-D kernel.  It stands where the paper puts its TF32 tensor-core path (Section
// 3.1.5: reduced-precision inputs, fp32 accumulation) and, like the fast kernel for narrow rows,
// keeps the labels exact: the error bound below is certified and points whose best scores fall
// inside it are settled by exact re-evaluation.
//
// Split: x ~ x0 + x1 with x0 = bf16(x), x1 = bf16(x - x0) - 16 significant bits, error at most
// 2^-16 |x| - and the same for the centroids; all four piece products are kept,
//     x.c ~ x0c0 + x0c1 + x1c0 + x1c1                (off by at most 2^-15 |x_d c_d| each feature).
// Why two pieces here and three for narrow rows: the rounding bound of the instructions themselves
// grows with their number (7 u of the magnitude each, u = 2^-24), and at 128 features the
// three-piece form (6 products per feature: 680 u) is certified only 2.2 times tighter than this
// one (4 products: 1480 u) while it needs half as many instructions again, LDS rows half as long
// again (256 centroids of 128 features would no longer fit a compute unit), and half as many
// point registers again.
//
// Layout: the 32x32x16 instruction contracts 16 values per lane pair - lane group g supplies
// k = 8g .. 8g+7 - and here the two groups take different FEATURES, as in the fp32 kernels: of a
// block of 16 features group g holds features 8g .. 8g+7.  A lane therefore keeps the pieces of
// half a row of its point (D/2 registers for two pieces) for the whole sweep, two points per lane
// (one in the streaming variant), and per block of 16 features two 16-byte LDS reads (its 8
// features of c0 and of c1) feed eight instructions (2 x 2 piece pairs, two points).  The centroid pieces are prepared once per call by
// split2_centroids_kernel, already in LDS image order, so staging is a plain copy.
//
// Per tile, each lane keeps the 16 scores of its best tile; at the end only the centroids whose
// scores lie inside the bound of the best are evaluated in direct-difference form from the fp32
// rows in memory (the point's row is fetched a second time for that; the pieces do not add up to
// it) - the winner always, up to three more - the two lanes of a point each covering the features
// they hold.  More candidates than that go to the refine kernel.
//
// What bounds it (measured): not the matrix unit, which is busy a quarter to a third of the time,
// but the two phases of a unit that wait for memory - the fetch of the rows and their second fetch
// with the winners' centroid rows - each as long as the sweep, with one other wave on the SIMD to
// fill the time.  All loads of a phase are therefore issued together, the compiler is kept from
// folding the second fetch into the first (which would hold the fp32 row in registers across the
// sweep), and where every tile is resident the rows of the NEXT unit are requested before the
// sweep of the current one (the STREAM variant: one point tile per unit).  Evaluating the
// distances with row-contiguous loads shared by the wave was tried and cost more vector
// instructions than it saved in waiting.
//
// Fault tolerance (Sections 2.3, 4): tiles of 30 centroids and two checksum rows, verification,
// location and correction as in the fp32 small-D kernel.  A checksum row is the sum of its 15
// centroids AFTER their reduction to two pieces, split in turn, so the truncation of the
// centroids cancels in the residual and only that of the one checksum row is left in it.
#include <cmath>
#include <type_traits>

#include "ftk_fast.h"
#include "ftk_internal.h"
#include "ftk_mma.h"
#include "ftk_smalld.h"

namespace ftk {

// Waves per workgroup (one workgroup per compute unit: two waves per SIMD, 256 registers each) and
// point tiles per wave.  Measured alternative for 128 features: twelve waves with one tile each
// (three per SIMD, 168 registers) - 10 % faster there, but twice the LDS reads per instruction and
// slower wherever the centroid image is staged in chunks.
constexpr int FW_WAVES = 8;
static constexpr int fw_pt(int nh) { (void)nh; return 2; }
// 16-byte units per centroid row in the LDS image: c0 then c1, 2*NH units each (NH blocks of 16
// features), plus one so that the 32 rows of a tile spread over the banks
static constexpr int fw_row_units(int nh) { return 4 * nh + 1; }

__device__ __forceinline__ void split2(float x, __bf16 &p0, __bf16 &p1)
{
    p0 = (__bf16)x;
    p1 = (__bf16)(x - (float)p0);  // the difference is exact
}

// Centroid pieces in LDS image order.  One thread per (row of the padded tiles, 8 features).
// Without checksums row 32T + i holds centroid 32T + i; with them a tile holds 30 centroids in the
// rows their accumulator registers read (register r of lane group g sits in row 8(r/4) + 4g + r%4)
// and the two rows of register 15 hold the sums of the groups' 15 two-piece centroids.
// Blocks beyond the image's (FT only): one wave per checksum row adds up the same 15 two-piece
// centroids and measures what the row loses when it is reduced to two pieces itself,
// delta = sum - (p0 + p1): the residual of a fault-free tile contains x . delta, which does not
// shrink with rounding noise, so the detection threshold carries ||x|| max ||delta|| (scal[1]).
template <int NH, bool FT>
__global__ __launch_bounds__(256) void split2_centroids_kernel(const float *C, int D, int K, int tiles_total, uint4 *img,
                                                               int image_blocks, double *scal)
{
    constexpr int SU = fw_row_units(NH);
    constexpr int NU = 2 * NH;
    if constexpr (FT) {
        if ((int)blockIdx.x >= image_blocks) {
            const int tg = ((int)blockIdx.x - image_blocks) * 4 + (int)(threadIdx.x >> 6);  // tile * 2 + lane group
            if (tg >= tiles_total * 2) return;
            const int lane = threadIdx.x & 63;
            const int j0 = 30 * (tg >> 1) + 15 * (tg & 1);
            float acc = 0.f;
            for (int d = lane; d < D; d += 64) {
                float sum = 0.f;
                for (int i = 0; i < 15 && j0 + i < K; ++i) {
                    __bf16 q0, q1;
                    split2(C[(size_t)(j0 + i) * D + d], q0, q1);
                    sum += (float)q0 + (float)q1;
                }
                __bf16 q0, q1;
                split2(sum, q0, q1);
                const float delta = sum - ((float)q0 + (float)q1);
                acc = fmaf(delta, delta, acc);
            }
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, 64);
            if (lane == 0 && acc > 0.f)
                atomicMax((unsigned long long *)(scal + 1), (unsigned long long)__double_as_longlong((double)sqrtf(acc)));
            return;
        }
    }
    const int rows = tiles_total * 32;
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= rows * NU) return;
    const int row = t / NU, u = t % NU;
    int j0 = row, nj = 1;
    if constexpr (FT) {
        const int T = row >> 5, lr = row & 31;
        const int gg = (lr >> 2) & 1, r = (lr >> 3) * 4 + (lr & 3);
        j0 = 30 * T + 15 * gg + (r < 15 ? r : 0);
        nj = r < 15 ? 1 : 15;
    }
    float sum[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) sum[e] = 0.f;
    for (int i = 0; i < nj; ++i) {
        const int j = j0 + i;
        if (j >= K) break;
        const float *src = C + (size_t)j * D;
        const floatx4 lo = load_frag<float, true>(src, 8 * u, D);
        const floatx4 hi = load_frag<float, true>(src, 8 * u + 4, D);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float v = e < 4 ? lo[e] : hi[e - 4];
            if (nj > 1) {  // a checksum row adds up what the matrix instructions will see
                __bf16 q0, q1;
                split2(v, q0, q1);
                v = (float)q0 + (float)q1;
            }
            sum[e] += v;
        }
    }
    bf16x8 p0, p1;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        __bf16 q0, q1;
        split2(sum[e], q0, q1);
        p0[e] = q0;
        p1[e] = q1;
    }
    uint4 *dst = img + (size_t)row * SU;  // tiles are 32 consecutive rows
    dst[u] = __builtin_bit_cast(uint4, p0);
    dst[NU + u] = __builtin_bit_cast(uint4, p1);
    if (u == 0) dst[2 * NU] = make_uint4(0u, 0u, 0u, 0u);  // the padding unit travels with the copy
}

// STREAM (every tile resident, no faults listed): one point tile per unit, and the rows of a wave's
// next unit are requested before the sweep of the current one, so that the first of the two
// memory phases of a unit passes under matrix work instead of in front of it.
template <int NH, bool FT, bool WHOLE, bool STREAM>
__global__ __launch_bounds__(FW_WAVES * 64, FW_WAVES / 4) void assign_fast_wide_kernel(FastArgs a)
{
    constexpr int THREADS = FW_WAVES * 64;
    constexpr int PT = STREAM ? 1 : fw_pt(NH);
    using M = Mma<float>;
    using G = TileGeom<FT>;
    constexpr int SU = fw_row_units(NH);
    constexpr int TU = 32 * SU;  // units per tile
    constexpr int NU = 2 * NH;   // 8-feature units per row; a lane holds unit 2*hb + g of block hb
    constexpr int RG = G::RG;
    constexpr int D8 = 16 * NH;
    extern __shared__ __align__(16) uint4 lds4[];
    uint4 *ldsC = lds4;                                                  // [tpc][TU]
    float *ldsH = reinterpret_cast<float *>(lds4 + (size_t)a.tpc * TU);  // [tpc*32] start values, (tile, group, register) order
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
    // largest ||delta|| of a checksum row (see split2_centroids_kernel), with room for ||x0 + x1|| over ||x||
    const float dnmax = FT ? 1.001f * (float)a.scal[1] : 0.f;
    const bool resident = a.nch == 1;
    int n_injected = 0, n_detected = 0, n_corrected = 0, n_recomputed = 0;
    float worst_resid = 0.f;

    for (int i = tid; i < SMALLD_LIST_CAP; i += THREADS) sh_wl[i] = -1;
    if (tid == 0) sh_wlcnt = 0;

    // stage tiles [ch*tpc, (ch+1)*tpc): a copy of the prepared image (eight 16-byte loads in flight
    // per thread, clamped instead of guarded) plus the accumulator start values.
    // Threads t0 .. t0 + nthr - 1 of the workgroup take part.
    auto stage_chunk = [&](int ch, int t0, int nthr) {
        const int tile0 = ch * a.tpc;
        const int ntile = min(a.tpc, a.tiles_total - tile0);
        const int ts = tid - t0;
        const uint4 *src = a.csplit + (size_t)tile0 * TU;
        const int n = ntile * TU;
        if (ts >= 0) {
            for (int base = ts; base < n; base += 8 * nthr) {
                uint4 f[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) f[u] = src[min(base + u * nthr, n - 1)];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (base + u * nthr < n) ldsC[base + u * nthr] = f[u];
            }
            for (int idx = ts; idx < ntile * 32; idx += nthr) {
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
        }
    };
    // With every tile resident the (only) chunk is staged inside the first unit of work and the two
    // halves of the workgroup start out of step: waves 0-3 fetch and split their points first and
    // wait while waves 4-7 copy the centroid image and only then fetch theirs.  Each SIMD holds one
    // wave of either half, so from then on one of its two waves multiplies while the other splits
    // or settles its points.
    bool staged = false;

    // this lane's half of point p's row: features 16hb + 8g .. + 7 of every block hb
    // WHOLE: rows as wide as the compiled variant need no guards; narrower ones take clamped
    // addresses and have the fragments beyond D (a multiple of 4) cleared afterwards (a variant of
    // its own: the guards are loop-invariant and would occupy registers for the whole kernel).
    // Either way no load sits in a branch of its own, so all of a row's loads are in flight at once.
    auto request_frags = [&](const float *row, floatx4 (&raw)[NU]) {
        if constexpr (WHOLE) {
#pragma unroll
            for (int u = 0; u < NU; ++u)
                raw[u] = *reinterpret_cast<const floatx4 *>(row + 16 * (u >> 1) + 8 * g + 4 * (u & 1));
        } else {
#pragma unroll
            for (int u = 0; u < NU; ++u) {
                const int off = 16 * (u >> 1) + 8 * g + 4 * (u & 1);
                const floatx4 v = load_frag_clamped<float, true>(row, off, D);
                const bool keep = off < D;
#pragma unroll
                for (int e = 0; e < 4; ++e) raw[u][e] = keep ? v[e] : 0.f;
            }
        }
    };
    auto request_row = [&](int64_t p, floatx4 (&raw)[NU]) { request_frags(a.X + p * D, raw); };
    // The same row fetched again after the sweep.  The index goes through an opaque copy: otherwise
    // the compiler recognises the addresses of the first fetch and, instead of loading twice, keeps
    // the fp32 row in registers across the sweep - the registers the pieces need.
    auto request_row_again = [&](int64_t p, floatx4 (&raw)[NU]) {
        asm volatile("" : "+v"(p));
        request_frags(a.X + p * D, raw);
    };

    // the fp32 rows of a unit between their request and their split: STREAM keeps them across units
    floatx4 raws_stream[STREAM ? PT : 1][STREAM ? NU : 1];
    bool have_rows = false;  // STREAM: the rows of the unit about to be processed have been requested

    // one unit of work of a wave: PT*32 points starting at p0, swept over all tiles and settled
    // (p0_next: the wave's next unit, or negative)
    auto process = [&](int64_t p0, int blk, int64_t p0_next) {
        uint4 b0[PT][NH], b1[PT][NH];  // pieces x0 and x1 of the lane's features, 8 per block
        float xn[PT];
        float tau[PT];
        float inv_tau[PT];
        int force_refine[PT];
        float rmax[PT];
        TileBest best[PT];
        floatx16 bacc[PT];  // the scores of this lane's best tile
        // fetch the rows (all loads of both tiles in flight together), split them into pieces;
        // norms, thresholds, empty records
        floatx4 raws_unit[STREAM ? 1 : PT][STREAM ? 1 : NU];
        auto &raws = [&]() -> auto & {
            if constexpr (STREAM) return raws_stream;
            else return raws_unit;
        }();
        auto request_unit = [&](int64_t q0) {
#pragma unroll
            for (int pt = 0; pt < PT; ++pt) {
                int64_t p = q0 + pt * 32 + col;
                if (p >= a.N) p = a.N - 1;
                request_row(p, raws[pt]);
            }
        };
        auto load_points = [&]() {
            if (!(STREAM && have_rows)) request_unit(p0);
#pragma unroll
            for (int pt = 0; pt < PT; ++pt) {
                const floatx4 (&raw)[NU] = raws[pt];
                float s = 0.f;
#pragma unroll
                for (int hb = 0; hb < NH; ++hb) {
                    bf16x8 q0, q1;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float v = raw[2 * hb + (e >> 2)][e & 3];
                        s = fmaf(v, v, s);
                        __bf16 u0, u1;
                        split2(v, u0, u1);
                        q0[e] = u0;
                        q1[e] = u1;
                    }
                    b0[pt][hb] = __builtin_bit_cast(uint4, q0);
                    b1[pt][hb] = __builtin_bit_cast(uint4, q1);
                }
                xn[pt] = s + __shfl_xor(s, 32, 64);
                tau[pt] = (float)a.ft_coef * (sqrtf(xn[pt]) * cmax + 0.5f * cmax2) + sqrtf(xn[pt]) * dnmax;
                inv_tau[pt] = 1.0f / tau[pt];
                force_refine[pt] = 0;
                rmax[pt] = 0.f;
                best[pt].m1 = best[pt].m2 = M::neg_inf();
                best[pt].t1 = 0;
#pragma unroll
                for (int r = 0; r < 16; ++r) bacc[pt][r] = M::neg_inf();
            }
            if (STREAM) {  // the next unit's rows travel while this one is swept
                have_rows = p0_next >= 0;
                if (have_rows) request_unit(p0_next);
            }
        };
        const bool head = !STREAM && resident && !staged && a.n_faults == 0;  // the out-of-step start (see above)
        const bool late = head && wave >= FW_WAVES / 2;
        if (!late) load_points();

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
            // the fragments of block hb + 1 are requested before the instructions of block hb are issued
            const uint4 *rowp = ldsC + (size_t)tl * TU + col * SU + g;
            uint4 n0 = rowp[0], n1 = rowp[NU];
#pragma unroll
            for (int hb = 0; hb < NH; ++hb) {
                const bf16x8 a0 = __builtin_bit_cast(bf16x8, n0);
                const bf16x8 a1 = __builtin_bit_cast(bf16x8, n1);
                if (hb + 1 < NH) {
                    n0 = rowp[2 * (hb + 1)];
                    n1 = rowp[NU + 2 * (hb + 1)];
                }
                // smallest products first; the PT accumulator chains are independent and interleave
#pragma unroll
                for (int pt = 0; pt < PT; ++pt)
                    accs[pt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, __builtin_bit_cast(bf16x8, b1[pt][hb]), accs[pt], 0, 0, 0);
#pragma unroll
                for (int pt = 0; pt < PT; ++pt)
                    accs[pt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, __builtin_bit_cast(bf16x8, b0[pt][hb]), accs[pt], 0, 0, 0);
#pragma unroll
                for (int pt = 0; pt < PT; ++pt)
                    accs[pt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, __builtin_bit_cast(bf16x8, b1[pt][hb]), accs[pt], 0, 0, 0);
#pragma unroll
                for (int pt = 0; pt < PT; ++pt)
                    accs[pt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, __builtin_bit_cast(bf16x8, b0[pt][hb]), accs[pt], 0, 0, 0);
            }
            // keep that order through instruction scheduling (which would otherwise move every read
            // next to its first use and leave one read in flight): start values and the first block,
            // then two reads ahead of each block's eight matrix instructions
            __builtin_amdgcn_sched_group_barrier(0x100, 6, 0);
#pragma unroll
            for (int hb = 0; hb + 1 < NH; ++hb) {
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 4 * PT, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 4 * PT, 0);
#pragma unroll
            for (int pt = 0; pt < PT; ++pt) {
                floatx16 acc = accs[pt];

                if constexpr (INJ) {  // fault injection (Section 2.1): flip one bit of one accumulator
                    for (int i = 0; i < nf; ++i) {
                        const ftk_fault f = sh_faults[i];
                        const int seq = (int)(f.tile % (unsigned)(a.tiles_total * PT));
                        if ((int)(f.wave % FW_WAVES) == wave && seq == T * PT + pt) {
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
                            // formed here on demand, in fp32 on the vector units, from the point's row
                            // in memory: this lane's features against its own group's weighted row and
                            // against the partner group's, the halves exchanged
                            float s2 = 0.f;
#pragma unroll
                            for (int r = 0; r < RG; ++r) s2 = fmaf((float)(r + 1), acc[r], s2);
                            int64_t p = p0 + pt * 32 + col;
                            if (p >= a.N) p = a.N - 1;
                            floatx4 xr[NU];
                            request_row_again(p, xr);
                            const float *v2 = a.chk_v2 + (size_t)(T * 2 + g) * D8;
                            const float *v2p = a.chk_v2 + (size_t)(T * 2 + (1 - g)) * D8;
                            float part = 0.f, cross = 0.f;
#pragma unroll
                            for (int u = 0; u < NU; ++u) {
                                const int off = 16 * (u >> 1) + 8 * g + 4 * (u & 1);
                                const floatx4 vo = *reinterpret_cast<const floatx4 *>(v2 + off);
                                const floatx4 vp = *reinterpret_cast<const floatx4 *>(v2p + off);
#pragma unroll
                                for (int e = 0; e < 4; ++e) {
                                    part = fmaf(xr[u][e], vo[e], part);
                                    cross = fmaf(xr[u][e], vp[e], cross);
                                }
                            }
                            const float ref2 = part + __shfl_xor(cross, 32, 64) - a.chk_s[(T * 2 + g) * 2 + 1];
                            const float delta = resid;
                            const float fpos = (s2 - ref2) / delta;
                            const float rpos = rintf(fpos);
                            const bool finite = (__float_as_uint(delta) & 0x7f800000u) != 0x7f800000u;
                            // the location is trusted only when the error stands far enough above the
                            // noise of the weighted sum; smaller detected errors are recomputed
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
                if (late) load_points();
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
            floatx4 xf[NU];  // the point's row again, in fp32: requested before anything else here
            request_row_again(live ? p : a.N - 1, xf);
            // scores inside `bound` of each other cannot be ordered: truncation to two pieces and
            // rounding of the instructions, plus (strict FT) an undetected error below the detection
            // threshold, which left its mark in the residual of its tile:
            // |error| <= |residual| + noise (taken as half the threshold)
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
                floatx4 cf[NU];
                request_frags(a.C + (size_t)(real ? j : 0) * D, cf);
                float d = 0.f;
#pragma unroll
                for (int u = 0; u < NU; ++u) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float t = xf[u][e] - cf[u][e];
                        d = fmaf(t, t, d);
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

    // Blocks of FW_WAVES units of PT*32 points.  With every tile resident and no faults listed the
    // waves are independent: each takes every gridDim-th block on its own, without barriers.
    // Otherwise the waves of a workgroup walk the blocks in step (chunks are staged, faults are
    // listed per block) and draw them from an atomic counter, one draw per block.
    int blk = blockIdx.x;
    if constexpr (STREAM) {
        stage_chunk(0, 0, THREADS);
        __syncthreads();
        staged = true;
        while (blk < a.nblocks) {
            const int nxt = blk + (int)gridDim.x;
            process(((int64_t)blk * FW_WAVES + wave) * (PT * 32), blk,
                    nxt < a.nblocks ? ((int64_t)nxt * FW_WAVES + wave) * (PT * 32) : -1);
            blk = nxt;
        }
    } else {
        while (blk < a.nblocks) {
            process(((int64_t)blk * FW_WAVES + wave) * (PT * 32), blk, -1);
            if (resident && a.n_faults == 0) {
                blk += (int)gridDim.x;
                continue;
            }
            __syncthreads();
            if (tid == 0) sh_next = (int)gridDim.x + atomicAdd(a.wl_count + 1, 1);
            __syncthreads();
            blk = sh_next;
        }
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
                atomicAdd(s, (unsigned long long)a.nblocks * FW_WAVES * PT * 64 * a.tiles_total);
            for (int i = 1; i < 5; ++i)
                if (v[i]) atomicAdd(s + i, (unsigned long long)v[i]);
            if (FT) {
                const unsigned long long mine = (unsigned long long)(fminf(worst_resid, 4000.f) * 1.0e6f);
                if (mine > *reinterpret_cast<volatile unsigned long long *>(s + 7)) atomicMax(s + 7, mine);
            }
        }
    }
}

// blocks of 16 features of the compiled variant that holds D features
static int fw_nh(int D)
{
    const int nh = (int)ceil_div(D, 16);
    return nh <= 3 ? 3 : (nh <= 4 ? 4 : (nh <= 6 ? 6 : 8));
}

size_t fast_wide_split_bytes(int D, int K)
{
    // tiles of 30 centroids when checksums are on
    return (size_t)ceil_div(K, 30) * 32 * fw_row_units(fw_nh(D)) * sizeof(uint4);
}

// Detection threshold: the rounding part has the form of the fp32 small-D tiles (15 scores against
// one checksum; the instructions sum 16 exact products and round once, so the coefficient is that
// of the three-piece kernel), and the kernel adds ||x|| max ||delta|| for what the two-piece
// checksum rows lose (measured per call by split2_centroids_kernel; at most 2^-16 of the sum of
// 15 centroids per feature, typically a tenth of that bound).
static constexpr double FW_FT_KAPPA = 1.0;
static double fw_ft_coef(int D)
{
    const double n = 15.0;
    return FW_FT_KAPPA * Mma<float>::kEps * n * (std::sqrt(n) + std::sqrt((double)D + 4.0));
}
static constexpr double FW_TRUNC_COEF = 1.001 * 15.0 / 65536.0;  // ||delta|| <= 2^-16 * 15 max ||c||

void plan_fast_wide(int64_t N, int D, int K, ftk_ft_mode ft, AssignPlan &p)
{
    const bool FT = ft != FTK_FT_OFF;
    const int nh = fw_nh(D);
    const int tiles_total = (int)ceil_div(K, FT ? 30 : 32);
    const int tile_bytes = 32 * fw_row_units(nh) * 16 + 32 * 4;
    // one workgroup per compute unit: it can stage nearly all of the 160 KB (156 KB)
    int tpc = (156 * 1024) / tile_bytes;
    if (tpc > tiles_total) tpc = tiles_total;
    tpc = (int)ceil_div(tiles_total, ceil_div(tiles_total, tpc));  // equal chunks
    p.variant = VAR_SMALLD;  // checksum rows and half-norm sums of the 30-centroid tiles
    p.TM = 32;
    p.TN = 32;
    p.PT = fw_pt(nh);
    p.KT = 1;
    p.waves = FW_WAVES;
    p.D8 = 16 * nh;
    p.DQ = nh;
    p.KC = 32;
    p.nkc = tiles_total;
    p.kch = tpc * 32;
    p.hcn_pad_inf = !FT;
    p.points_per_wg = p.waves * p.PT * 32;
    p.workgroups = ceil_div(N, p.points_per_wg);
    p.grid = (int)(p.workgroups < 256 ? p.workgroups : 256);
    p.tiles_per_wave = tiles_total * p.PT;
    p.regs_per_tile = 16;
    p.lds_bytes = (size_t)tpc * tile_bytes;
    p.ft_coef = fw_ft_coef(D);
    p.ft_trunc_coef = FT ? FW_TRUNC_COEF : 0.0;
    // two scores, each: truncation of both operands to two pieces (2^-15 = 512 u of the magnitude),
    // 4*nh instructions at 7 u, and 2 u for the fp32 evaluation of the magnitude itself
    p.band_coef = 2.0 * (512.0 + 28.0 * nh + 4.0) * Mma<float>::kEps;
}

template <int NH, bool FT>
static void launch_fast_wide_t(const FastArgs &a, const AssignPlan &p, hipStream_t st)
{
    const int rows = a.tiles_total * 32;
    const int image_blocks = (int)ceil_div((int64_t)rows * 2 * NH, 256);
    const int delta_blocks = FT ? (int)ceil_div(a.tiles_total * 2, 4) : 0;
    hipLaunchKernelGGL((split2_centroids_kernel<NH, FT>), dim3(image_blocks + delta_blocks), dim3(256), 0, st, a.C, a.D,
                       a.K, a.tiles_total, const_cast<uint4 *>(a.csplit), image_blocks, const_cast<double *>(a.scal));
    // every tile resident and no faults listed: the streaming variant, one point tile per unit
    // (measured: 13 % faster at 128 features, 5 % at 96, and 10-25 % with checksums at every width -
    // one tile's verification state instead of two keeps the sweep loop free of spills; without
    // checksums up to 64 features the two-tile units are 4 % ahead)
    const bool stream = a.nch == 1 && a.n_faults == 0 && (NH >= 6 || FT);
    FastArgs b = a;
    int grid = p.grid;
    if (stream) {
        const int64_t blocks = ceil_div(a.N, (int64_t)FW_WAVES * 32);
        b.nblocks = (int)blocks;
        grid = (int)(blocks < 256 ? blocks : 256);
    }
    const dim3 g((unsigned)grid), t(FW_WAVES * 64);
    if (a.D == 16 * NH) {
        if (stream) hipLaunchKernelGGL((assign_fast_wide_kernel<NH, FT, true, true>), g, t, p.lds_bytes, st, b);
        else hipLaunchKernelGGL((assign_fast_wide_kernel<NH, FT, true, false>), g, t, p.lds_bytes, st, b);
    } else {
        if (stream) hipLaunchKernelGGL((assign_fast_wide_kernel<NH, FT, false, true>), g, t, p.lds_bytes, st, b);
        else hipLaunchKernelGGL((assign_fast_wide_kernel<NH, FT, false, false>), g, t, p.lds_bytes, st, b);
    }
}

ftk_status launch_assign_fast_wide(const AssignCall &c, const AssignPlan &p, const Workspace &w, hipStream_t st)
{
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
#define FTK_LAUNCH_FAST_WIDE(NHV)                         \
    do {                                                  \
        if (FT) launch_fast_wide_t<NHV, true>(a, p, st);  \
        else launch_fast_wide_t<NHV, false>(a, p, st);    \
    } while (0)
    switch (p.DQ) {
    case 3: FTK_LAUNCH_FAST_WIDE(3); break;
    case 4: FTK_LAUNCH_FAST_WIDE(4); break;
    case 6: FTK_LAUNCH_FAST_WIDE(6); break;
    default: FTK_LAUNCH_FAST_WIDE(8); break;
    }
#undef FTK_LAUNCH_FAST_WIDE
    FTK_TRY_HIP(hipGetLastError());
    return FTK_OK;
}

}  // namespace ftk
