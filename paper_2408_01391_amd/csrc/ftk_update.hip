// Centroid update, Eq. (2): per-cluster sums and counts, then the averaging pass.
//
// The paper's kernel (Section 3.1.2) has every thread add its point into the global sums with
// floating-point atomics, whose result depends on the order in which the adds land.  Here the
// sums are accumulated in 64-bit FIXED POINT: every coordinate is scaled by a power of two
// fixed from max|x| and the number of points a workgroup handles so that no workgroup sum can
// overflow, rounded once to an integer, and added with integer atomics.  Integer addition is
// associative, so the sums - and the centroids - are bitwise identical from run to run
// whatever the schedule, and the only rounding is the one quantisation per coordinate
// (<= 2^-(62 - ceil(log2 rows_per_workgroup)) relative to max|x|, below 2^-45 for the
// workloads here).  Workgroup sums are flushed into a two-limb global accumulator (high part
// and low 24 bits separately), so the global sum cannot overflow either.
//
// Accumulation is privatised in LDS: a workgroup owns a block of points and a [Ks x Ds] slice
// of the sum matrix that fits 64 KB, adds into it with LDS atomics, and flushes the non-zero
// cells to the global matrix with one integer atomic each.  Feature slices partition the
// columns of X and cluster slices partition its rows by label, so X is read once overall.
#include <type_traits>

#include "ftk_internal.h"
#include "ftk_mma.h"

namespace ftk {

constexpr int UPD_CELLS = 8192;  // int64 cells per workgroup slice (64 KB)
constexpr int UPD_TARGET_WGS = 256;  // one 1024-thread workgroup per CU: every extra table is one more slab to write and re-read
constexpr int UPD_THREADS = 1024;  // threads per workgroup of the LDS path: many waves per 64 KB table hide the HBM latency

struct UpdatePlan {
    int Ks, Ds, nks, nds, tx_log2;
    int64_t rows_per_chunk;
    int chunks;
    bool aligned;
};

// Row chunks of the LDS path never exceed UPD_TARGET_WGS or one per 64 rows; with S
// slices of at most UPD_CELLS cells covering the K*D table, chunks <= UPD_TARGET_WGS / S, hence
// chunks * K * D <= UPD_TARGET_WGS * UPD_CELLS whenever more than one chunk is used.
int64_t update_slab_chunks_max(int64_t N)
{
    const int64_t by_rows = ceil_div(N, 64);
    return by_rows < UPD_TARGET_WGS ? (by_rows < 1 ? 1 : by_rows) : UPD_TARGET_WGS;
}
// walkers of the label-sorted path: one per RED_ROWS_PER_LANE_MIN rows at most
int64_t update_walkers_max(int64_t N) { return ceil_div(N, 64) + 1; }
int64_t update_slab_cells_max(int64_t N, int D, int K)
{
    const int64_t cells = (int64_t)K * D;
    const int64_t cap = (int64_t)UPD_TARGET_WGS * UPD_CELLS;
    int64_t v = update_slab_chunks_max(N) * cells;
    if (v > cap) v = cap;
    return v > cells ? v : cells;
}

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
    const int ppr = u.aligned ? (u.Ds + E - 1) / E : u.Ds;  // pieces per row slice
    int l2 = 0;
    while ((1 << l2) < ppr && l2 < 8) ++l2;
    u.tx_log2 = l2;
    // a workgroup takes UPD_THREADS >> tx_log2 rows per pass; at least 16 passes (and 64 rows) per
    // chunk, so that long rows of a mid-sized problem still spread over all CUs
    int64_t min_rows = (int64_t)16 * (UPD_THREADS >> l2);
    if (min_rows > UPD_THREADS) min_rows = UPD_THREADS;
    if (min_rows < 64) min_rows = 64;
    int chunks = UPD_TARGET_WGS / slices;
    if (chunks < 1) chunks = 1;
    if (chunks > ceil_div(N, min_rows)) chunks = (int)ceil_div(N, min_rows);
    u.chunks = chunks;
    u.rows_per_chunk = ceil_div(N, chunks);
    return u;
}

__global__ void update_zero_kernel(unsigned long long *sums, int64_t n, int32_t *counts, int K)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) sums[i] = 0ull;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < K; i += stride) counts[i] = 0;
}

constexpr int UPD_LIMB_BITS = 24;

// scale = 2^(62 - ceil(log2 rows) - (ilogb(absmax) + 1)): rows * max|x| * scale <= 2^62.
// rows is taken as at least 2048, which keeps every scaled coordinate below 2^51 so that the
// conversion below is valid.
__device__ __forceinline__ double fixed_point_scale(double absmax, int64_t rows)
{
    int L = 11;
    while (((int64_t)1 << L) < rows) ++L;
    if (!(absmax > 0.0) || !(absmax < __builtin_huge_val())) return 1.0;
    return ldexp(1.0, 62 - L - (ilogb(absmax) + 1));
}

// round(x * scale) as a 64-bit integer, for |x * scale| < 2^51: adding 1.5 * 2^52 in one fused
// operation leaves the rounded integer in the low mantissa bits (one rounding, to nearest even).
__device__ __forceinline__ long long to_fixed(double x, double scale)
{
    constexpr double MAGIC = 6755399441055744.0;  // 1.5 * 2^52
    return __double_as_longlong(fma(x, scale, MAGIC)) - __double_as_longlong(MAGIC);
}

// ---- dual modular redundancy (paper Sections 2.3 and 4: the memory-bound update is protected
// by duplicating its arithmetic and comparing) ------------------------------------------------
// The loads are not duplicated (a flipped bit in memory is outside the paper's fault model,
// Section 2.1); every arithmetic result that leaves a register is produced twice, from operands
// the compiler must treat as unrelated, and the two results are compared as integers.
__device__ __forceinline__ double dmr_copy(double v)
{
    asm volatile("" : "+v"(v));  // opaque: prevents the two instruction streams from being merged
    return v;
}

// mean = (hi * 2^LIMB + lo) / scale / n, rounded once to T.  DMR: evaluated twice from operands the
// compiler must treat as unrelated; if the two results differ a third evaluation decides.
template <typename T, bool DMR>
__device__ __forceinline__ T fixed_point_mean(long long hi, long long lo, double inv, int n, int *detected)
{
    const double total = (double)hi * (double)(1ll << UPD_LIMB_BITS) + (double)lo;
    T m = (T)((total * inv) / (double)n);
    if constexpr (DMR) {
        const double total2 = dmr_copy((double)hi) * (double)(1ll << UPD_LIMB_BITS) + dmr_copy((double)lo);
        const T m2 = (T)((total2 * dmr_copy(inv)) / dmr_copy((double)n));
        if (m != m2) {
            const double total3 = dmr_copy(dmr_copy((double)hi)) * (double)(1ll << UPD_LIMB_BITS) + dmr_copy(dmr_copy((double)lo));
            const T m3 = (T)((total3 * dmr_copy(dmr_copy(inv))) / dmr_copy(dmr_copy((double)n)));
            m = (m3 == m2) ? m2 : m;
            *detected += 1;
        }
    }
    return m;
}

struct UpdateFtArgs {
    const ftk_fault *faults;  // device; addressed as (workgroup, wave, step, element, lane, bit)
    int n_faults;
    int mode;                 // ftk_ft_mode
    ftk_ft_stats *stats;
};
constexpr int UPD_MAX_FAULTS = 4;  // injected faults honoured per workgroup

// faults aimed at this workgroup -> LDS; returns how many (uniform)
__device__ __forceinline__ int stage_faults(const UpdateFtArgs &ft, int wg, ftk_fault *sh_faults, int *sh_nf,
                                            int nthreads)
{
    if (ft.n_faults <= 0) return 0;
    if (threadIdx.x == 0) *sh_nf = 0;
    __syncthreads();
    for (int i = threadIdx.x; i < ft.n_faults; i += nthreads) {
        if ((int)ft.faults[i].workgroup == wg) {
            const int slot = atomicAdd(sh_nf, 1);
            if (slot < UPD_MAX_FAULTS) sh_faults[slot] = ft.faults[i];
        }
    }
    __syncthreads();
    return min(*sh_nf, UPD_MAX_FAULTS);
}

__device__ __forceinline__ void add_stat(ftk_ft_stats *stats, int field, int n)
{
    if (stats && n) atomicAdd(reinterpret_cast<unsigned long long *>(stats) + field, (unsigned long long)n);
}
enum { STAT_INJECTED = 1, STAT_DETECTED = 2, STAT_CORRECTED = 3, STAT_RECOMPUTED = 4, STAT_UNCORRECTABLE = 5 };

template <typename T, bool ALIGNED, bool DMR>
__global__ __launch_bounds__(UPD_THREADS) void update_accumulate_kernel(
    const T *X, const int32_t *labels, int64_t N, int D, int K, const double *absmax_p,
    long long *slabs, int32_t *cslabs, int Ks, int Ds, int nds, int tx_log2,
    int64_t rows_per_chunk, int64_t scale_rows, int accumulate, UpdateFtArgs ft)
{
    using F = typename Mma<T>::frag_t;
    constexpr int E = ALIGNED ? Mma<T>::E : 1;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    unsigned long long *cell = reinterpret_cast<unsigned long long *>(lds_raw);
    // table rows are padded by one cell: a row of Ds 8-byte cells is a whole number of LDS bank
    // rounds for the slice widths in use (8, 32, 128 features), so without the pad the lanes of a
    // wave - several point rows with different labels, same feature offsets - would all hit the
    // same banks
    const int Dp = Ds + 1;
    int *cnt = reinterpret_cast<int *>(cell + (size_t)Ks * Dp);
    __shared__ unsigned long long sh_sum[4];  // [0] table total, [1] shadow total, [2] count total, [3] shadow rows
    __shared__ int sh_nf;
    __shared__ ftk_fault sh_faults[UPD_MAX_FAULTS];

    const int tid = threadIdx.x;
    const int slice = blockIdx.y;
    const int ds_i = slice % nds, ks_i = slice / nds;
    const int d0 = ds_i * Ds, k0 = ks_i * Ks;
    const int dn = min(Ds, D - d0);  // features in this slice
    const int kn = min(Ks, K - k0);
    // fp32 data: 24-bit mantissas leave ample room, one limb scaled for the whole of N;
    // fp64 data: scale for the rows that meet in this workgroup's table only (scale_rows: one
    // chunk of rows, times the number of batches when the table is accumulated over several
    // launches) and flush into two limbs
    const double scale = fixed_point_scale(*absmax_p, scale_rows);
    const double scale2 = dmr_copy(scale);
    const int TX = 1 << tx_log2, TY = UPD_THREADS >> tx_log2;
    const int tx = tid & (TX - 1), ty = tid >> tx_log2;
    const int ppr = (dn + E - 1) / E;
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_chunk;
    const int64_t r1 = r0 + rows_per_chunk < N ? r0 + rows_per_chunk : N;
    const int nf = stage_faults(ft, (int)blockIdx.x, sh_faults, &sh_nf, UPD_THREADS);
    int n_injected = 0;

    // DMR: the conversion is done twice and compared on the spot; the accumulation into the LDS
    // table is shadowed by a per-thread running total of everything the thread added (second
    // instruction stream, registers only).  After the pass the table's total must equal the sum
    // of the shadows, and the member counts the number of rows counted; if not, the workgroup
    // clears its table and repeats the pass (injection, which models a transient error, is not
    // repeated).
    constexpr int ATTEMPTS = DMR ? 2 : 1;
    for (int attempt = 0; attempt < ATTEMPTS; ++attempt) {
        for (int i = tid; i < Ks * Dp; i += UPD_THREADS) cell[i] = 0ull;
        for (int i = tid; i < Ks; i += UPD_THREADS) cnt[i] = 0;
        if (tid < 4) sh_sum[tid] = 0ull;
        __syncthreads();
        unsigned long long shadow = 0ull;  // wraps like the table does
        unsigned shadow_rows = 0;
        int step = 0;

        // UNR rows per thread and step: the label loads, then the point loads, are issued together
        // before any LDS atomic, so several HBM requests per thread are in flight
        constexpr int UNR = 4;
        // When the slice holds every cluster the point loads do not depend on the labels and go out
        // together with them (ALLK); otherwise only rows whose label falls into the slice are read,
        // one memory latency after their labels.
        auto pass = [&](auto allk_tag) {
        constexpr bool ALLK = decltype(allk_tag)::value;
        for (int64_t row0 = r0 + ty; row0 < r1; row0 += (int64_t)TY * UNR, ++step) {
            int lab[UNR];
            bool ok[UNR];
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                const int64_t row = row0 + (int64_t)u * TY;
                lab[u] = row < r1 ? labels[row] - k0 : -1;
            }
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                ok[u] = (unsigned)lab[u] < (unsigned)kn;
                if (ok[u] && tx == 0 && ds_i == 0) {
                    atomicAdd(&cnt[lab[u]], 1);
                    if (DMR) shadow_rows += 1;
                }
            }
            // injected soft error (fault model of Section 2.1): one bit of one converted operand of
            // this step, after the comparison and before it is accumulated
            unsigned long long flip[UNR];
#pragma unroll
            for (int u = 0; u < UNR; ++u) flip[u] = 0ull;
            int flip_e = -1;
            if (nf > 0 && attempt == 0) {
                for (int i = 0; i < nf; ++i) {
                    const ftk_fault f = sh_faults[i];
                    // the addressed thread, moved onto the lane of its row that owns a piece
                    const int ft_id = (int)(f.wave % (UPD_THREADS / 64)) * 64 + (int)(f.lane & 63);
                    if ((ft_id >> tx_log2) == ty && ((ft_id & (TX - 1)) % ppr) == tx && (int)f.tile == step) {
                        flip[f.reg % UNR] = 1ull << (f.bit & 63);
                        flip_e = (int)((f.reg / UNR) % E);
                    }
                }
            }
            for (int pc = tx; pc < ppr; pc += TX) {
                F f[UNR];
#pragma unroll
                for (int u = 0; u < UNR; ++u) {
                    const int64_t row = row0 + (int64_t)u * TY;
                    if (ALLK ? row < r1 : ok[u]) {
                        if constexpr (ALIGNED) f[u] = *reinterpret_cast<const F *>(X + row * D + d0 + pc * E);
                        else f[u][0] = X[row * D + d0 + pc];
                    }
                }
#pragma unroll
                for (int u = 0; u < UNR; ++u) {
                    if (ok[u]) {
                        unsigned long long *dst = cell + (size_t)lab[u] * Dp + pc * E;
#pragma unroll
                        for (int e = 0; e < E; ++e) {
                            const double x = (double)f[u][e];
                            long long v = to_fixed(x, scale);
                            if constexpr (DMR) {
                                long long v2 = to_fixed(dmr_copy(x), scale2);
                                if (v != v2) {  // conversion disagrees: do it a third time and keep the majority
                                    const long long v3 = to_fixed(dmr_copy(dmr_copy(x)), scale2);
                                    v = (v3 == v2) ? v2 : v;
                                    v2 = v;
                                }
                                shadow += (unsigned long long)v2;
                            }
                            if (flip[u] != 0ull && e == flip_e && pc == tx) {
                                v = (long long)((unsigned long long)v ^ flip[u]);
                                n_injected += 1;
                            }
                            atomicAdd(dst + e, (unsigned long long)v);
                        }
                    }
                }
            }
        }
        };
        if (kn == K)
            pass(std::true_type{});
        else
            pass(std::false_type{});
        __syncthreads();
        if constexpr (DMR) {
            unsigned long long tsum = 0ull, csum = 0ull;
            for (int i = tid; i < Ks * Dp; i += UPD_THREADS) tsum += cell[i];
            for (int i = tid; i < Ks; i += UPD_THREADS) csum += (unsigned long long)(unsigned)cnt[i];
            // wave totals first, then one LDS atomic per wave and word
            unsigned long long v4[4] = {tsum, shadow, csum, (unsigned long long)shadow_rows};
#pragma unroll
            for (int w4 = 0; w4 < 4; ++w4)
#pragma unroll
                for (int mask = 1; mask < 64; mask <<= 1) v4[w4] += __shfl_xor(v4[w4], mask, 64);
            if ((tid & 63) == 0)
                for (int w4 = 0; w4 < 4; ++w4) atomicAdd(&sh_sum[w4], v4[w4]);
            __syncthreads();
            const bool good = sh_sum[0] == sh_sum[1] && sh_sum[2] == sh_sum[3];
            __syncthreads();
            if (good) break;
            if (tid == 0) {
                add_stat(ft.stats, STAT_DETECTED, 1);
                if (ft.mode >= FTK_FT_CORRECT) add_stat(ft.stats, attempt == 0 ? STAT_RECOMPUTED : STAT_UNCORRECTABLE, 1);
            }
            if (ft.mode < FTK_FT_CORRECT) break;  // detect only: the corrupted table is flushed
        }
    }
    if (nf > 0) {
#pragma unroll
        for (int mask = 1; mask < 64; mask <<= 1) n_injected += __shfl_xor(n_injected, mask, 64);
        if ((tid & 63) == 0) add_stat(ft.stats, STAT_INJECTED, n_injected);
    }
    // Flush with plain stores into this row chunk's table in global memory (every cell of the
    // slice, zeros included, so the tables need no clearing).  Device-wide atomics on one shared
    // table cost a memory-side transaction per cell and workgroup; the tables are summed by the
    // averaging kernel instead, in integers, so the result is still independent of any order.
    // (`accumulate`: a later batch of the same Lloyd iteration adds to what its predecessors left;
    // a table cell belongs to one workgroup, so this needs no atomics either.)
    long long *slab = slabs + (int64_t)blockIdx.x * ((int64_t)K * D);
    for (int i = tid; i < kn * Ds; i += UPD_THREADS) {
        const int k = i / Ds, d = i - k * Ds;
        if (d < dn) {
            long long *dst = slab + (int64_t)(k0 + k) * D + d0 + d;
            *dst = (accumulate ? *dst : 0ll) + (long long)cell[k * Dp + d];
        }
    }
    if (ds_i == 0)
        for (int i = tid; i < kn; i += UPD_THREADS) {
            int32_t *dst = cslabs + (int64_t)blockIdx.x * K + k0 + i;
            *dst = (accumulate ? *dst : 0) + cnt[i];
        }
}

// Sum of the per-chunk tables and averaging pass ("the last kernel", Section 3.1.1) in one:
// C_j = sum_j / count_j, rounded once; a cluster without points keeps its previous centroid.
// A workgroup owns RF_CELLS consecutive cells; its RF_GROUPS thread groups each add every
// RF_GROUPS-th table (coalesced reads, several in flight), the partial sums meet in LDS.
// fp64 data: the tables were scaled for one chunk's rows, so the sum over chunks is carried in
// two limbs.
constexpr int RF_CELLS = 32, RF_GROUPS = 32;
// DMR: two sets of table sums are kept and compared before the partial sums are combined; a
// mismatch is settled by a third pass.
template <typename T, bool DMR>
__global__ __launch_bounds__(RF_CELLS * RF_GROUPS) void update_reduce_finalize_kernel(
    const long long *slabs, const int32_t *cslabs, int chunks, int64_t scale_rows, int D,
    int K, const double *absmax_p, T *C, int32_t *counts, ftk_ft_stats *stats)
{
    constexpr bool TWO_LIMB = sizeof(T) == 8;
    __shared__ long long sh_hi[RF_GROUPS][RF_CELLS], sh_lo[RF_GROUPS][RF_CELLS];
    __shared__ int sh_cnt[RF_GROUPS][RF_CELLS];
    const int ci = threadIdx.x % RF_CELLS, grp = threadIdx.x / RF_CELLS;
    const int64_t cells = (int64_t)K * D;
    const int64_t cell0 = (int64_t)blockIdx.x * RF_CELLS;
    const int64_t cell = cell0 + ci;
    // member counts of the rows this workgroup touches (at most RF_CELLS): thread ci <-> row
    const int row0 = (int)(cell0 / D);
    const int64_t last_cell = cell0 + RF_CELLS - 1 < cells ? cell0 + RF_CELLS - 1 : cells - 1;
    const int nrows = (int)(last_cell / D) - row0 + 1;
    // one pass over the tables; under DMR every value loaded is added into two sets of sums (the
    // second through an opaque copy), which are compared before the partial sums are combined
    int c = 0, c2 = 0, detected = 0;
    long long hi = 0, lo = 0, hi2 = 0, lo2 = 0;
#pragma unroll 4
    for (int ch = grp; ch < chunks; ch += RF_GROUPS) {
        if (ci < nrows) {
            int n = cslabs[(int64_t)ch * K + row0 + ci];
            c += n;
            if constexpr (DMR) {
                asm volatile("" : "+v"(n));
                c2 += n;
            }
        }
        if (cell < cells) {
            long long v = slabs[(int64_t)ch * cells + cell];
            if (TWO_LIMB) {
                hi += v >> UPD_LIMB_BITS;                      // floor
                lo += v & ((1ll << UPD_LIMB_BITS) - 1);        // >= 0
            } else {
                lo += v;
            }
            if constexpr (DMR) {
                asm volatile("" : "+v"(v));
                if (TWO_LIMB) {
                    hi2 += v >> UPD_LIMB_BITS;
                    lo2 += v & ((1ll << UPD_LIMB_BITS) - 1);
                } else {
                    lo2 += v;
                }
            }
        }
    }
    if constexpr (DMR) {
        if (hi != hi2 || lo != lo2 || c != c2) {  // settle by a third, separate pass
            long long hi3 = 0, lo3 = 0;
            int c3 = 0;
            for (int ch = grp; ch < chunks; ch += RF_GROUPS) {
                if (ci < nrows) c3 += cslabs[(int64_t)ch * K + row0 + ci];
                if (cell < cells) {
                    const long long v = slabs[(int64_t)ch * cells + cell];
                    if (TWO_LIMB) {
                        hi3 += v >> UPD_LIMB_BITS;
                        lo3 += v & ((1ll << UPD_LIMB_BITS) - 1);
                    } else {
                        lo3 += v;
                    }
                }
            }
            hi = hi3;
            lo = lo3;
            c = c3;
            detected += 1;
        }
    }
    sh_hi[grp][ci] = hi;
    sh_lo[grp][ci] = lo;
    sh_cnt[grp][ci] = c;
    __syncthreads();
    if (grp == 0) {
        for (int g2 = 1; g2 < RF_GROUPS; ++g2) {
            hi += sh_hi[g2][ci];
            lo += sh_lo[g2][ci];
            c += sh_cnt[g2][ci];
        }
        sh_cnt[0][ci] = c;  // row totals, read back below by the threads of other cells
    }
    __syncthreads();
    if (grp == 0) {
        if (ci < nrows) {
            // every row's first cell lies in exactly one workgroup: that one publishes the count
            const int64_t first = (int64_t)(row0 + ci) * D;
            if (first >= cell0 && first <= last_cell) counts[row0 + ci] = c;
        }
        if (cell < cells) {
            const int n = sh_cnt[0][(int)(cell / D) - row0];
            if (n > 0) {
                const double inv = 1.0 / fixed_point_scale(*absmax_p, scale_rows);
                C[cell] = fixed_point_mean<T, DMR>(hi, lo, inv, n, &detected);
            }
        }
    }
    if (DMR && detected) {
        add_stat(stats, STAT_DETECTED, detected);
        add_stat(stats, STAT_RECOMPUTED, detected);
    }
}

// ======================= label-sorted path (rows of at least one cache line) =================
// Points are first bucketed by label (counting sort: histogram, scan, scatter); the reduction
// then walks the sorted order, where a lane sees long runs of one label and can keep the
// running sum of its features in registers, touching memory only when the label changes.
// No LDS and no atomics in the inner loop; the order inside a bucket is whatever the scatter
// produced, which is irrelevant because fixed-point sums do not depend on it.

constexpr int SORT_CHUNK = 4096;       // points per workgroup in histogram / scatter
constexpr int SORT_PER_THREAD = SORT_CHUNK / 256;
constexpr int SORT_MAX_K_LDS = 8192;   // clusters whose per-workgroup histogram fits LDS

// counts[k] += number of points of this chunk with label k  (counts zeroed beforehand)
__global__ __launch_bounds__(256) void sort_hist_kernel(const int32_t *labels, int64_t N, int K, int32_t *counts)
{
    extern __shared__ int lh[];
    const bool use_lds = K <= SORT_MAX_K_LDS;
    if (use_lds) {
        for (int k = threadIdx.x; k < K; k += 256) lh[k] = 0;
        __syncthreads();
    }
    const int64_t base = (int64_t)blockIdx.x * SORT_CHUNK;
#pragma unroll 4
    for (int i = 0; i < SORT_PER_THREAD; ++i) {
        const int64_t p = base + i * 256 + threadIdx.x;
        if (p < N) {
            const int lab = labels[p];
            if ((unsigned)lab < (unsigned)K) {
                if (use_lds) atomicAdd(&lh[lab], 1);
                else atomicAdd(&counts[lab], 1);
            }
        }
    }
    if (use_lds) {
        __syncthreads();
        for (int k = threadIdx.x; k < K; k += 256)
            if (lh[k]) atomicAdd(&counts[k], lh[k]);
    }
}

// cursor[k] = exclusive prefix sum of counts (one workgroup, fixed order)
__global__ __launch_bounds__(1024) void sort_scan_kernel(const int32_t *counts, int K, int32_t *cursor)
{
    __shared__ int sh[1024];
    __shared__ int carry;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (int k0 = 0; k0 < K; k0 += 1024) {
        const int k = k0 + threadIdx.x;
        const int v = k < K ? counts[k] : 0;
        sh[threadIdx.x] = v;
        __syncthreads();
        for (int off = 1; off < 1024; off <<= 1) {
            const int t = threadIdx.x >= off ? sh[threadIdx.x - off] : 0;
            __syncthreads();
            sh[threadIdx.x] += t;
            __syncthreads();
        }
        if (k < K) cursor[k] = carry + sh[threadIdx.x] - v;
        __syncthreads();
        if (threadIdx.x == 1023) carry += sh[1023];
        __syncthreads();
    }
    if (threadIdx.x == 0) cursor[K] = carry;  // number of validly labelled points; not touched by the scatter
}

// sorted_idx / sorted_lab: point indices and labels grouped by label.  Each workgroup ranks its
// points inside LDS, reserves one range per label with a single global atomic, then writes.
__global__ __launch_bounds__(256) void sort_scatter_kernel(const int32_t *labels, int64_t N, int K, int32_t *cursor,
                                                           int32_t *sorted_idx, int32_t *sorted_lab)
{
    extern __shared__ int lh[];  // [K] local counts, then reused as local bases
    const bool use_lds = K <= SORT_MAX_K_LDS;
    const int64_t base = (int64_t)blockIdx.x * SORT_CHUNK;
    int lab[SORT_PER_THREAD], rank[SORT_PER_THREAD];
    if (use_lds) {
        for (int k = threadIdx.x; k < K; k += 256) lh[k] = 0;
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < SORT_PER_THREAD; ++i) {
        const int64_t p = base + i * 256 + threadIdx.x;
        lab[i] = -1;
        rank[i] = 0;
        if (p < N) {
            const int l = labels[p];
            if ((unsigned)l < (unsigned)K) {
                lab[i] = l;
                rank[i] = use_lds ? atomicAdd(&lh[l], 1) : atomicAdd(&cursor[l], 1);
            }
        }
    }
    if (use_lds) {
        __syncthreads();
        for (int k = threadIdx.x; k < K; k += 256) {
            const int c = lh[k];
            lh[k] = c ? atomicAdd(&cursor[k], c) : 0;
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < SORT_PER_THREAD; ++i) {
        if (lab[i] >= 0) {
            const int pos = (use_lds ? lh[lab[i]] : 0) + rank[i];
            sorted_idx[pos] = (int32_t)(base + i * 256 + threadIdx.x);
            sorted_lab[pos] = lab[i];
        }
    }
}

constexpr int RED_ROWS_PER_LANE_MAX = 256;  // most sorted positions one walker covers
constexpr int RED_ROWS_PER_LANE_MIN = 64;

// Walk the sorted order.  lpr_log2: lanes per row (power of two); a wave holds 64/lpr "walkers"
// (row groups), each covering rows_per_lane consecutive sorted positions; blockIdx.y selects the
// slice of 64*E features when a row is wider than one wave.
//
// Where the sums go when a run of one label ends - without any atomics:
//   * the label's whole segment lies inside this walker's range: the walker owns the result and
//     stores it straight into `sums`;
//   * the segment started before the range (then the run is the walker's first) or continues
//     after it (then it is the last): the partial sum goes to the walker's slot 0 resp. 1,
//     tagged with the label, and the averaging kernel adds the slots of the walkers a segment
//     touches.  (cursor[k] is the end of segment k after the scatter, cursor[K] their total.)
template <typename T, bool ALIGNED, bool DMR, bool NT = false>
__global__ __launch_bounds__(256) void sorted_reduce_kernel(const T *X, const int32_t *sorted_idx,
                                                            const int32_t *sorted_lab, const int32_t *cursor,
                                                            int K, int64_t N, int D, int lpr_log2, int rows_per_lane,
                                                            int64_t n_walkers, const double *absmax_p,
                                                            long long *sums, long long *slot_val,
                                                            int32_t *slot_lab, UpdateFtArgs ft)
{
    using F = typename Mma<T>::frag_t;
    constexpr int E = ALIGNED ? Mma<T>::E : 1;
    constexpr bool TWO_LIMB = sizeof(T) == 8;
    constexpr int UNR = 8;
    __shared__ int sh_nf;
    __shared__ ftk_fault sh_faults[UPD_MAX_FAULTS];
    const int lane = threadIdx.x & 63;
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lpr = 1 << lpr_log2, gpw = 64 >> lpr_log2;
    const int group = lane >> lpr_log2, piece = lane & (lpr - 1);
    const int d0 = (blockIdx.y * 64 + piece) * E;  // first feature of this lane
    const bool lane_on = d0 < D;
    // fp32: one limb scaled for the whole of N; fp64: scaled for one walker's rows, two limbs later
    const double scale = fixed_point_scale(*absmax_p, TWO_LIMB ? RED_ROWS_PER_LANE_MAX : N);
    const double scale2 = dmr_copy(scale);
    const int64_t walker = wave * gpw + group;
    const int64_t n_sorted = cursor[K];
    const int64_t s_begin = min(n_sorted, walker * (int64_t)rows_per_lane);
    const int64_t s_end = min(n_sorted, (walker + 1) * (int64_t)rows_per_lane);
    const int nf = blockIdx.y == 0 ? stage_faults(ft, (int)blockIdx.x, sh_faults, &sh_nf, 256) : 0;
    int n_injected = 0, n_detected = 0, n_recomputed = 0, n_uncorrectable = 0;  // per lane (runs end in divergent flow)

    // DMR: a second set of running sums is fed by a second conversion of the same loaded values;
    // the two sets are compared as integers whenever a run ends, i.e. before anything leaves the
    // registers.  On a mismatch the lane walks its run again (both streams) and stores that.
    long long acc[E], acc2[E];
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] = acc2[e] = 0;
    int cur = -1;
    int slot_label0 = -1, slot_label1 = -1;
    int64_t run_start = s_begin;  // sorted position of the first row of the current run
    auto flush = [&](int64_t run_end) {
        if constexpr (DMR) {
            bool bad = false;
            if (cur >= 0 && lane_on) {
#pragma unroll
                for (int e = 0; e < E; ++e) bad |= acc[e] != acc2[e];
            }
            if (__builtin_expect(__any(bad), 0)) {
                n_detected += bad ? 1 : 0;
                if (ft.mode >= FTK_FT_CORRECT) {
                    bool ok = true;
                    if (bad) {
                        long long r1[E], r2[E];
#pragma unroll
                        for (int e = 0; e < E; ++e) r1[e] = r2[e] = 0;
                        for (int64_t s = run_start; s < run_end; ++s) {
                            const int64_t row = sorted_idx[s];
#pragma unroll
                            for (int e = 0; e < E; ++e) {
                                const double x = (d0 + e < D) ? (double)X[row * D + d0 + e] : 0.0;
                                r1[e] += to_fixed(x, scale);
                                r2[e] += to_fixed(dmr_copy(x), scale2);
                            }
                        }
#pragma unroll
                        for (int e = 0; e < E; ++e) {
                            ok = ok && r1[e] == r2[e];
                            acc[e] = r1[e];
                        }
                    }
                    n_recomputed += (bad && ok) ? 1 : 0;
                    n_uncorrectable += (bad && !ok) ? 1 : 0;
                }
            }
        }
        if (cur >= 0) {
            const int64_t seg_a = cur ? cursor[cur - 1] : 0, seg_b = cursor[cur];
            const bool interior = seg_a >= s_begin && seg_b <= s_end;
            const int slot = seg_a < s_begin ? 0 : 1;
            if (!interior) {
                if (slot == 0) slot_label0 = cur;
                else slot_label1 = cur;
            }
            if (lane_on) {
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    if (d0 + e < D) {
                        if (interior) {
                            long long *dst = sums + 2 * ((int64_t)cur * D + d0 + e);
                            if (TWO_LIMB) {
                                dst[0] = acc[e] >> UPD_LIMB_BITS;                      // floor
                                dst[1] = acc[e] & ((1ll << UPD_LIMB_BITS) - 1);        // >= 0
                            } else {
                                dst[1] = acc[e];
                            }
                        } else {
                            slot_val[(walker * 2 + slot) * D + d0 + e] = acc[e];
                        }
                    }
                    acc[e] = 0;
                    if (DMR) acc2[e] = 0;
                }
            }
        }
    };
    // software pipeline: the index / label pairs of the next batch are fetched while the point
    // rows of the current batch are in flight
    int lab_n[UNR];
    int64_t row_n[UNR];
    auto fetch_keys = [&](int64_t s0) {
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int64_t s = s0 + u;
            const bool in = s < s_end;
            lab_n[u] = in ? sorted_lab[s] : -1;
            row_n[u] = in ? sorted_idx[s] : 0;
        }
    };
    fetch_keys(s_begin);
    int step = 0;
    for (int64_t s0 = s_begin; s0 < s_end; s0 += UNR, ++step) {
        int lab[UNR];
        F f[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            lab[u] = lab_n[u];
            if (lab[u] >= 0 && lane_on) {
                // NT: X far larger than the 256 MB memory-side cache and read exactly once - streaming
                // (non-temporal) loads then sustain 12-15 % more than ordinary ones on this device;
                // for an X that the preceding assignment left in that cache they are slower
                if constexpr (ALIGNED && NT) f[u] = __builtin_nontemporal_load(reinterpret_cast<const F *>(X + row_n[u] * D + d0));
                else if constexpr (ALIGNED) f[u] = *reinterpret_cast<const F *>(X + row_n[u] * D + d0);
                else f[u][0] = X[row_n[u] * D + d0];
            }
        }
        fetch_keys(s0 + UNR);
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            if (lab[u] >= 0) {
                if (lab[u] != cur) {
                    flush(s0 + u);
                    cur = lab[u];
                    run_start = s0 + u;
                }
                if (lane_on) {
#pragma unroll
                    for (int e = 0; e < E; ++e) {
                        const double x = (double)f[u][e];
                        acc[e] += to_fixed(x, scale);
                        if (DMR) acc2[e] += to_fixed(dmr_copy(x), scale2);
                    }
                }
            }
        }
        // injected soft error (fault model of Section 2.1): one bit of one running sum of the first
        // instruction stream, after this step's additions
        if (__builtin_expect(nf > 0, 0)) {
            for (int i = 0; i < nf; ++i) {
                const ftk_fault fl = sh_faults[i];
                if ((int)(fl.wave & 3) == (int)(threadIdx.x >> 6) && (int)fl.tile == step) {
                    // the addressed lane, moved onto a lane of its row group that owns features
                    const int fl_lane = (int)(fl.lane & 63);
                    const int pa = min(lpr, (D + E - 1) / E);
                    const bool me = group == (fl_lane >> lpr_log2) && piece == (fl_lane & (lpr - 1)) % pa &&
                                    lane_on && cur >= 0;
#pragma unroll
                    for (int e = 0; e < E; ++e)
                        if (me && (int)(fl.reg % E) == e)
                            acc[e] = (long long)((unsigned long long)acc[e] ^ (1ull << (fl.bit & 63)));
                    n_injected += me ? 1 : 0;
                }
            }
        }
    }
    flush(s_end);
    // slot tags (the same from every feature slice)
    if (piece == 0 && walker < n_walkers) {
        slot_lab[walker * 2 + 0] = slot_label0;
        slot_lab[walker * 2 + 1] = slot_label1;
    }
    if (ft.stats && (DMR || nf > 0)) {
#pragma unroll
        for (int mask = 1; mask < 64; mask <<= 1) {
            n_injected += __shfl_xor(n_injected, mask, 64);
            n_detected += __shfl_xor(n_detected, mask, 64);
            n_recomputed += __shfl_xor(n_recomputed, mask, 64);
            n_uncorrectable += __shfl_xor(n_uncorrectable, mask, 64);
        }
    }
    if (ft.stats && lane == 0) {
        add_stat(ft.stats, STAT_INJECTED, n_injected);
        add_stat(ft.stats, STAT_DETECTED, n_detected);
        add_stat(ft.stats, STAT_RECOMPUTED, n_recomputed);
        add_stat(ft.stats, STAT_UNCORRECTABLE, n_uncorrectable);
    }
}

// Averaging pass of the label-sorted path: per cell, the sum stored by the owning walker (zero if
// none) plus the tagged slots of the walkers the label's segment touches; then the mean.  Same
// tiling idea as update_reduce_finalize_kernel: thread groups stride over the walkers.
// a segment touches few walkers (its length / rows per walker + 2), so few thread groups per cell
constexpr int SF_CELLS = 32, SF_GROUPS = 8;
template <typename T, bool DMR>
__global__ __launch_bounds__(SF_CELLS * SF_GROUPS) void sorted_finalize_kernel(
    const long long *sums, const long long *slot_val, const int32_t *slot_lab, const int32_t *cursor,
    int rows_per_lane, int64_t N, int D, int K, const double *absmax_p, T *C, ftk_ft_stats *stats)
{
    constexpr bool TWO_LIMB = sizeof(T) == 8;
    __shared__ long long sh_hi[SF_GROUPS][SF_CELLS], sh_lo[SF_GROUPS][SF_CELLS];
    const int ci = threadIdx.x % SF_CELLS, grp = threadIdx.x / SF_CELLS;
    const int64_t cells = (int64_t)K * D;
    const int64_t cell = (int64_t)blockIdx.x * SF_CELLS + ci;
    const bool on = cell < cells;
    const int k = on ? (int)(cell / D) : 0;
    const int d = on ? (int)(cell - (int64_t)k * D) : 0;
    const int64_t seg_a = k ? cursor[k - 1] : 0, seg_b = cursor[k];
    const int n = (int)(seg_b - seg_a);
    long long hi = 0, lo = 0, hi2 = 0, lo2 = 0;
    int detected = 0;
    if (on && n > 0) {
        if (grp == 0) {
            hi = hi2 = sums[2 * cell];
            lo = lo2 = sums[2 * cell + 1];
        }
        const int64_t w_lo = seg_a / rows_per_lane, w_hi = (seg_b - 1) / rows_per_lane;
        // tags and values are loaded unconditionally (unused slots hold stale data that the tag
        // deselects): no load depends on another, so several walkers are in flight per thread
#pragma unroll 4
        for (int64_t w = w_lo + grp; w <= w_hi; w += SF_GROUPS) {
#pragma unroll
            for (int slot = 0; slot < 2; ++slot) {
                const int tag = slot_lab[w * 2 + slot];
                long long v = slot_val[(w * 2 + slot) * D + d];
                v = tag == k ? v : 0ll;
                if (TWO_LIMB) {
                    hi += v >> UPD_LIMB_BITS;
                    lo += v & ((1ll << UPD_LIMB_BITS) - 1);
                } else {
                    lo += v;
                }
                if constexpr (DMR) {
                    asm volatile("" : "+v"(v));
                    if (TWO_LIMB) {
                        hi2 += v >> UPD_LIMB_BITS;
                        lo2 += v & ((1ll << UPD_LIMB_BITS) - 1);
                    } else {
                        lo2 += v;
                    }
                }
            }
        }
        if constexpr (DMR) {
            if (hi != hi2 || lo != lo2) {  // settle by a third pass
                long long hi3 = grp == 0 ? sums[2 * cell] : 0, lo3 = grp == 0 ? sums[2 * cell + 1] : 0;
                for (int64_t w = w_lo + grp; w <= w_hi; w += SF_GROUPS)
                    for (int slot = 0; slot < 2; ++slot)
                        if (slot_lab[w * 2 + slot] == k) {
                            const long long v = slot_val[(w * 2 + slot) * D + d];
                            if (TWO_LIMB) {
                                hi3 += v >> UPD_LIMB_BITS;
                                lo3 += v & ((1ll << UPD_LIMB_BITS) - 1);
                            } else {
                                lo3 += v;
                            }
                        }
                hi = hi3;
                lo = lo3;
                detected += 1;
            }
        }
    }
    sh_hi[grp][ci] = hi;
    sh_lo[grp][ci] = lo;
    __syncthreads();
    if (grp == 0 && on && n > 0) {
        for (int g2 = 1; g2 < SF_GROUPS; ++g2) {
            hi += sh_hi[g2][ci];
            lo += sh_lo[g2][ci];
        }
        const double inv = 1.0 / fixed_point_scale(*absmax_p, TWO_LIMB ? RED_ROWS_PER_LANE_MAX : N);
        C[cell] = fixed_point_mean<T, DMR>(hi, lo, inv, n, &detected);
    }
    if (DMR && detected) {
        add_stat(stats, STAT_DETECTED, detected);
        add_stat(stats, STAT_RECOMPUTED, detected);
    }
}

// Launch geometry of the pass that accumulates the sums (the one faults are injected into).
struct UpdateLaunch {
    bool sorted_path;
    UpdatePlan u;
    // sorted path
    int lpr_log2, rows_per_lane, pieces, E;
    int64_t n_walkers;
    dim3 rgrid;
};
static UpdateLaunch plan_update_launch(ftk_dtype dtype, const void *X, int64_t N, int D, int K)
{
    UpdateLaunch L;
    L.u = plan_update(dtype, X, N, D, K);
    const size_t esz = dtype == FTK_F32 ? 4 : 8;
    // Rows of at least half a cache line gather efficiently, and the label-sorted path streams
    // them at nearly the HBM rate - but it is six kernels with a fixed cost of about 45 us, and the
    // two-kernel LDS path reads X exactly once as long as one slice holds every cluster (K <= 256:
    // the slices then split the features only).  Measured crossovers (both paths forced, N = 2^17
    // .. 2^20, fp32 and fp64): with all clusters resident the LDS path wins up to about 0.75 GB of
    // X (e.g. 2^20 x 128, K = 256: 128 against 159 us; 2^17 x 1024, K = 128: 141 against 180 us)
    // and loses beyond (LDS atomics per element against a streaming reduction: 2^20 x 256: 253
    // against 224 us); with the clusters split over several slices it re-reads X once per slice
    // and wins only for small tables on data that stay in the memory-side cache.
    const double x_bytes = (double)N * D * esz;
    const bool small_table = (L.u.nks == 1 && x_bytes < 805306368.0) ||
                             ((int64_t)K * D <= 4 * UPD_CELLS && x_bytes < 268435456.0);
    L.sorted_path = (size_t)D * esz >= 64 && N >= 65536 && !small_table;
    if (g_tuning.update_path >= 0) L.sorted_path = g_tuning.update_path == 1;
    L.E = L.u.aligned ? (dtype == FTK_F32 ? 4 : 2) : 1;
    L.pieces = (int)ceil_div(D, L.E);
    L.lpr_log2 = 0;
    while ((1 << L.lpr_log2) < L.pieces && L.lpr_log2 < 6) ++L.lpr_log2;
    const int gpw = 64 >> L.lpr_log2;
    // about 2048 waves where N allows (run ends cost only plain stores, so parallelism is free)
    int64_t rpl = N / ((int64_t)gpw * 2048);
    if (rpl < RED_ROWS_PER_LANE_MIN) rpl = RED_ROWS_PER_LANE_MIN;
    if (rpl > RED_ROWS_PER_LANE_MAX) rpl = RED_ROWS_PER_LANE_MAX;
    L.rows_per_lane = (int)rpl;
    L.n_walkers = ceil_div(N, L.rows_per_lane);
    const int64_t waves = ceil_div(L.n_walkers, gpw);
    L.rgrid = dim3((unsigned)ceil_div(waves, 4), (unsigned)ceil_div(L.pieces, 64));
    return L;
}

void update_geometry(ftk_dtype dtype, bool aligned16, int64_t N, int D, int K, ftk_geometry *out)
{
    const UpdateLaunch L = plan_update_launch(dtype, aligned16 ? nullptr : (const void *)1, N, D, K);
    if (L.sorted_path) {
        out->workgroups = L.rgrid.x;
        out->waves_per_workgroup = 4;
        out->tiles_per_wave = (uint32_t)ceil_div(L.rows_per_lane, 8);
        out->regs_per_tile = (uint32_t)L.E;
    } else {
        const int TY = UPD_THREADS >> L.u.tx_log2;
        out->workgroups = (uint32_t)L.u.chunks;
        out->waves_per_workgroup = UPD_THREADS / 64;
        out->tiles_per_wave = (uint32_t)ceil_div(L.u.rows_per_chunk, (int64_t)TY * 4);
        out->regs_per_tile = (uint32_t)(4 * L.E);
    }
    out->lanes = 64;
    out->bits = 64;
}

ftk_status launch_update(ftk_dtype dtype, const void *X, const int32_t *labels, int64_t N, int D,
                         int K, void *C, int32_t *counts, const double *absmax, const Workspace &w,
                         ftk_ft_mode ft_mode, const ftk_fault *faults, int n_faults, ftk_ft_stats *stats,
                         hipStream_t st)
{
    const UpdateLaunch L = plan_update_launch(dtype, X, N, D, K);
    const UpdatePlan &u = L.u;
    const int64_t cells = (int64_t)K * D;
    unsigned long long *sums = reinterpret_cast<unsigned long long *>(w.fx_sums);
    const bool dmr = ft_mode != FTK_FT_OFF;
    UpdateFtArgs fa;
    fa.faults = faults;
    fa.n_faults = n_faults;
    fa.mode = (int)ft_mode;
    fa.stats = stats;
    if (L.sorted_path) {
        {
            const int blocks = (int)(ceil_div(cells, 256) < 1024 ? ceil_div(cells, 256) : 1024);
            hipLaunchKernelGGL(update_zero_kernel, dim3(blocks), dim3(256), 0, st, sums, 2 * cells, counts, K);
        }
        const int chunks = (int)ceil_div(N, SORT_CHUNK);
        const size_t hl = K <= SORT_MAX_K_LDS ? (size_t)K * 4 : 0;
        hipLaunchKernelGGL(sort_hist_kernel, dim3(chunks), dim3(256), hl, st, labels, N, K, counts);
        hipLaunchKernelGGL(sort_scan_kernel, dim3(1), dim3(1024), 0, st, counts, K, w.sort_cursor);
        hipLaunchKernelGGL(sort_scatter_kernel, dim3(chunks), dim3(256), hl, st, labels, N, K, w.sort_cursor,
                           w.sort_idx, w.sort_lab);
        dim3 rblock(256);
        long long *slot_val = reinterpret_cast<long long *>(w.upd_slab);
        int32_t *slot_lab = w.upd_cslab;
        if (L.n_walkers > update_walkers_max(N)) {
            set_error("internal: %lld walkers exceed the workspace bound", (long long)L.n_walkers);
            return FTK_EINVAL;
        }
        const bool stream_x = (double)N * D * (dtype == FTK_F32 ? 4 : 8) >= 1073741824.0;  // >= 1 GiB
#define FTK_LAUNCH_RED(T, AL, DM, ...)                                                                  \
    hipLaunchKernelGGL((sorted_reduce_kernel<T, AL, DM, ##__VA_ARGS__>), L.rgrid, rblock, 0, st, (const T *)X, w.sort_idx, \
                       w.sort_lab, w.sort_cursor, K, N, D, L.lpr_log2, L.rows_per_lane, L.n_walkers, absmax, \
                       reinterpret_cast<long long *>(sums), slot_val, slot_lab, fa)
#define FTK_LAUNCH_RED_T(T)                                \
    do {                                                   \
        if (u.aligned && dmr && stream_x) FTK_LAUNCH_RED(T, true, true, true);   \
        else if (u.aligned && stream_x) FTK_LAUNCH_RED(T, true, false, true);    \
        else if (u.aligned && dmr) FTK_LAUNCH_RED(T, true, true);  \
        else if (u.aligned) FTK_LAUNCH_RED(T, true, false);        \
        else if (dmr) FTK_LAUNCH_RED(T, false, true);              \
        else FTK_LAUNCH_RED(T, false, false);                      \
    } while (0)
        if (dtype == FTK_F32) FTK_LAUNCH_RED_T(float);
        else FTK_LAUNCH_RED_T(double);
#undef FTK_LAUNCH_RED_T
#undef FTK_LAUNCH_RED
        {
            const int blocks = (int)ceil_div(cells, SF_CELLS);
#define FTK_LAUNCH_FIN(T, DM)                                                                              \
    hipLaunchKernelGGL((sorted_finalize_kernel<T, DM>), dim3(blocks), dim3(SF_CELLS * SF_GROUPS), 0, st,  \
                       reinterpret_cast<const long long *>(sums), slot_val, slot_lab, w.sort_cursor,       \
                       L.rows_per_lane, N, D, K, absmax, (T *)C, stats)
            if (dtype == FTK_F32) {
                if (dmr) FTK_LAUNCH_FIN(float, true);
                else FTK_LAUNCH_FIN(float, false);
            } else {
                if (dmr) FTK_LAUNCH_FIN(double, true);
                else FTK_LAUNCH_FIN(double, false);
            }
#undef FTK_LAUNCH_FIN
        }
    } else {
        if (u.chunks > update_slab_chunks_max(N) || (int64_t)u.chunks * cells > update_slab_cells_max(N, D, K)) {
            set_error("internal: update tables exceed the workspace bound (chunks %d)", u.chunks);
            return FTK_EINVAL;
        }
        const size_t lds = (size_t)u.Ks * (u.Ds + 1) * 8 + (size_t)u.Ks * 4;
        dim3 grid(u.chunks, u.nds * u.nks), block(UPD_THREADS);
        long long *slabs = reinterpret_cast<long long *>(w.upd_slab);
        const int64_t scale_rows = dtype == FTK_F64 ? u.rows_per_chunk : N;
#define FTK_LAUNCH_ACC(T, AL, DM)                                                                      \
    hipLaunchKernelGGL((update_accumulate_kernel<T, AL, DM>), grid, block, lds, st, (const T *)X, labels, \
                       N, D, K, absmax, slabs, w.upd_cslab, u.Ks, u.Ds, u.nds, u.tx_log2, u.rows_per_chunk, \
                       scale_rows, 0, fa)
#define FTK_LAUNCH_ACC_T(T)                                \
    do {                                                   \
        if (u.aligned && dmr) FTK_LAUNCH_ACC(T, true, true);       \
        else if (u.aligned) FTK_LAUNCH_ACC(T, true, false);        \
        else if (dmr) FTK_LAUNCH_ACC(T, false, true);              \
        else FTK_LAUNCH_ACC(T, false, false);                      \
    } while (0)
        if (dtype == FTK_F32) FTK_LAUNCH_ACC_T(float);
        else FTK_LAUNCH_ACC_T(double);
#undef FTK_LAUNCH_ACC_T
#undef FTK_LAUNCH_ACC
        const int blocks = (int)ceil_div(cells, RF_CELLS);
#define FTK_LAUNCH_RF(T, DM)                                                                                  \
    hipLaunchKernelGGL((update_reduce_finalize_kernel<T, DM>), dim3(blocks), dim3(RF_CELLS * RF_GROUPS), 0, st, \
                       slabs, w.upd_cslab, u.chunks, scale_rows, D, K, absmax, (T *)C, counts, stats)
        if (dtype == FTK_F32) {
            if (dmr) FTK_LAUNCH_RF(float, true);
            else FTK_LAUNCH_RF(float, false);
        } else {
            if (dmr) FTK_LAUNCH_RF(double, true);
            else FTK_LAUNCH_RF(double, false);
        }
#undef FTK_LAUNCH_RF
    }
    FTK_TRY_HIP(hipGetLastError());
    return FTK_OK;
}

// ---- update accumulated over batches of rows (the batched Lloyd step) ------------------------
// The per-workgroup LDS tables of one batch are added to the tables in global memory its
// predecessors left (plain read-modify-write: a table belongs to one workgroup), and the
// reduce-and-average kernel runs once after the last batch.  The plan is the one of a full batch;
// a shorter last batch only changes the rows per workgroup.
BatchedUpdatePlan plan_update_batched(ftk_dtype dtype, const void *X, int64_t N, int64_t batch_rows, int D, int K)
{
    const UpdatePlan u = plan_update(dtype, X, batch_rows < N ? batch_rows : N, D, K);
    BatchedUpdatePlan b;
    b.Ks = u.Ks;
    b.Ds = u.Ds;
    b.nks = u.nks;
    b.nds = u.nds;
    b.tx_log2 = u.tx_log2;
    b.chunks = u.chunks;
    b.aligned = u.aligned;
    const int64_t nbatch = ceil_div(N, batch_rows);
    b.scale_rows = dtype == FTK_F64 ? u.rows_per_chunk * nbatch : N;
    b.ok = u.chunks <= update_slab_chunks_max(N) && (int64_t)u.chunks * K * D <= update_slab_cells_max(N, D, K);
    return b;
}

ftk_status launch_update_batch(ftk_dtype dtype, const void *Xb, const int32_t *labels_b, int64_t nb, int D, int K,
                               const double *absmax, const Workspace &w, const BatchedUpdatePlan &b, bool first,
                               hipStream_t st)
{
    const size_t lds = (size_t)b.Ks * (b.Ds + 1) * 8 + (size_t)b.Ks * 4;
    dim3 grid(b.chunks, b.nds * b.nks), block(UPD_THREADS);
    long long *slabs = reinterpret_cast<long long *>(w.upd_slab);
    const int64_t rows_per_chunk = ceil_div(nb, b.chunks);
    UpdateFtArgs fa;
    fa.faults = nullptr;
    fa.n_faults = 0;
    fa.mode = (int)FTK_FT_OFF;
    fa.stats = nullptr;
#define FTK_LAUNCH_ACC(T, AL)                                                                             \
    hipLaunchKernelGGL((update_accumulate_kernel<T, AL, false>), grid, block, lds, st, (const T *)Xb, labels_b, \
                       nb, D, K, absmax, slabs, w.upd_cslab, b.Ks, b.Ds, b.nds, b.tx_log2, rows_per_chunk,  \
                       b.scale_rows, first ? 0 : 1, fa)
    if (dtype == FTK_F32) {
        if (b.aligned) FTK_LAUNCH_ACC(float, true);
        else FTK_LAUNCH_ACC(float, false);
    } else {
        if (b.aligned) FTK_LAUNCH_ACC(double, true);
        else FTK_LAUNCH_ACC(double, false);
    }
#undef FTK_LAUNCH_ACC
    FTK_TRY_HIP(hipGetLastError());
    return FTK_OK;
}

ftk_status launch_update_batched_finalize(ftk_dtype dtype, int D, int K, const double *absmax, void *C,
                                          int32_t *counts, const Workspace &w, const BatchedUpdatePlan &b,
                                          hipStream_t st)
{
    const int64_t cells = (int64_t)K * D;
    const int blocks = (int)ceil_div(cells, RF_CELLS);
    const long long *slabs = reinterpret_cast<const long long *>(w.upd_slab);
    if (dtype == FTK_F32)
        hipLaunchKernelGGL((update_reduce_finalize_kernel<float, false>), dim3(blocks), dim3(RF_CELLS * RF_GROUPS), 0, st,
                           slabs, w.upd_cslab, b.chunks, b.scale_rows, D, K, absmax, (float *)C, counts, nullptr);
    else
        hipLaunchKernelGGL((update_reduce_finalize_kernel<double, false>), dim3(blocks), dim3(RF_CELLS * RF_GROUPS), 0, st,
                           slabs, w.upd_cslab, b.chunks, b.scale_rows, D, K, absmax, (double *)C, counts, nullptr);
    FTK_TRY_HIP(hipGetLastError());
    return FTK_OK;
}

}  // namespace ftk
