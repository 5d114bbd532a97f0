/*
 * ftkmeans.h -- C boundary of the MI355X (gfx950) K-means hot path.
 *
 * One Lloyd iteration of K-means (paper Section 2) is
 *     assignment  label_i = argmin_j || X_i - C_j ||_2                       (Eq. 1)
 *     update      C_j     = mean of the points with label j                  (Eq. 2)
 * The assignment is evaluated through the expansion of Section 3.1.2,
 *     || x - c ||^2 = sum_d x_d^2 + sum_d c_d^2 - 2 sum_d x_d c_d,
 * whose last term is a dense [N x D] by [D x K] contraction on the matrix cores with the
 * per-point argmin fused into its epilogue (Sections 3.1.3-3.1.5), optionally protected by
 * the online checksum scheme of Sections 2.3 and 4 (detect, locate, correct one corrupted
 * accumulator element per checked tile before the argmin reads it).
 *
 * Conventions common to every call
 *   - N points, D features, K clusters.  X is [N x D], C is [K x D], both row-major and
 *     contiguous, element type given by `dtype`.
 *   - Every array pointer is a DEVICE pointer owned by the caller unless marked (host).
 *     The library allocates no device memory: scratch comes from `workspace`, which must
 *     hold at least ftk_workspace_bytes(...) bytes and be 256-byte aligned.  Workspace
 *     contents need not survive between calls.
 *   - Calls only enqueue work on `hip_stream` (a hipStream_t; NULL = the default stream)
 *     and return without waiting, except where stated.  Calls that share a workspace must be
 *     ordered on one stream.
 *   - Distances are SQUARED Euclidean distances (the square root is dropped, Section 3.1.2).
 *   - Exact ties go to the lowest centroid index.  An empty cluster keeps its centroid.
 *   - Errors are reported by return code, never by abort; ftk_last_error() gives the text of
 *     the last failure on the calling thread.  Argument, alignment and workspace errors are
 *     found before anything is enqueued; a HIP runtime failure (FTK_EDEVICE) may leave kernels of
 *     the failed call on the stream, and the outputs are then undefined.
 */
#ifndef FTKMEANS_H
#define FTKMEANS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FTK_OK = 0,
    FTK_EINVAL = 1,        /* bad shape, NULL pointer, unknown enum value            */
    FTK_EALIGN = 2,        /* a pointer is not aligned to its element size / 256 B   */
    FTK_EWORKSPACE = 3,    /* workspace missing or too small                         */
    FTK_EDEVICE = 4,       /* a HIP runtime call failed or the device is not gfx950  */
    FTK_EUNCORRECTABLE = 5 /* reserved: never returned; see ftk_ft_stats.uncorrectable   */
} ftk_status;

typedef enum { FTK_F32 = 0, FTK_F64 = 1 } ftk_dtype;

/* Fault-tolerance mode of the contraction (Section 4).
 *   OFF     : no checksums.
 *   DETECT  : checksums carried and verified, mismatches only counted.
 *   CORRECT : a mismatching tile is repaired in place from its location-encoded checksums
 *             (Section 4.1); if the location cannot be decoded the tile is recomputed.
 *             As in the paper, an error smaller than the detection threshold (the rounding
 *             noise of the checksum comparison) passes unnoticed; it can change the label
 *             of a point only if that point's two best scores are closer than the threshold.
 *   STRICT  : CORRECT, and in addition every point whose decision an error below the threshold
 *             could have changed - its best scores are closer than the largest checksum
 *             residual seen for that point plus half the threshold for rounding noise - is
 *             settled by exact re-evaluation, so the labels equal those of a fault-free run
 *             whatever single error occurred per checked tile.  Costs the exact re-evaluation
 *             of those points.  This is the mode the benchmark reports overhead for. */
typedef enum { FTK_FT_OFF = 0, FTK_FT_DETECT = 1, FTK_FT_CORRECT = 2, FTK_FT_STRICT = 3 } ftk_ft_mode;

/* One injected soft error (fault model of Section 2.1): flip `bit` of accumulator register
 * `reg` of lane `lane`, in the `tile`-th output tile that wave `wave` of workgroup
 * `workgroup` finishes, right after its matrix instructions and before verification.
 * Fields other than `workgroup` are reduced modulo the extents ftk_assign_geometry reports,
 * so every descriptor is valid; a workgroup index beyond the grid never fires. */
typedef struct {
    uint32_t workgroup, wave, tile, reg, lane, bit;
} ftk_fault;

/* Counters accumulated (atomically added to) by ftk_kmeans_assign; zero them beforehand. */
typedef struct {
    uint64_t tiles_checked;  /* per-lane-group checksum comparisons made                  */
    uint64_t injected;       /* fault descriptors that fired                              */
    uint64_t detected;       /* checksum mismatches above the threshold                   */
    uint64_t corrected;      /* repaired from the decoded location                        */
    uint64_t recomputed;     /* location not decodable -> tile recomputed                 */
    uint64_t uncorrectable;  /* update step only: a recomputed pass mismatched again; the
                                assignment recomputes outside the matrix path and never
                                produces it                                               */
    uint64_t refined;        /* points whose best scores were closer than the rounding-
                                error bound and were re-evaluated exactly by the refine
                                kernel                                                    */
    uint64_t max_residual_ppm; /* largest fault-free checksum residual seen, in millionths
                                of the detection threshold (maximised, not added)        */
} ftk_ft_stats;

/* Launch geometry of the assignment kernel for a problem, for building fault lists. */
typedef struct {
    uint32_t workgroups, waves_per_workgroup, tiles_per_wave, regs_per_tile, lanes, bits;
} ftk_geometry;

/* Bytes of workspace sufficient for any of the three calls below on this problem. */
size_t ftk_workspace_bytes(ftk_dtype dtype, int64_t N, int32_t D, int32_t K, ftk_ft_mode ft);

ftk_status ftk_assign_geometry(ftk_dtype dtype, int64_t N, int32_t D, int32_t K, ftk_ft_mode ft,
                               ftk_geometry *out /* (host) */);

/* (host) The two error scales of the assignment kernel chosen for a problem (16-byte aligned X
 * and C assumed), both as multiples of B_i = ||x_i|| max_j||c_j|| + max_j||c_j||^2 / 2, in units
 * of the score s_ij = x_i.c_j - ||c_j||^2/2 (half a squared distance):
 *   detect_coef : checksum detection threshold of Section 2.3 / 4.1 ("a defined threshold"): a
 *                 corrupted score is noticed when the error exceeds detect_coef * B_i; 0 with
 *                 fault tolerance off.  In FTK_FT_CORRECT a smaller error passes and can move
 *                 point i only between centroids whose squared distances differ by less than
 *                 2 * detect_coef * B_i; in FTK_FT_STRICT it cannot move it at all.
 *   band_coef   : scores closer than band_coef * B_i are not ordered by the matrix path but
 *                 settled by exact re-evaluation. */
ftk_status ftk_ft_thresholds(ftk_dtype dtype, int64_t N, int32_t D, int32_t K, ftk_ft_mode ft,
                             double *detect_coef /* (host) */, double *band_coef /* (host) */);

/* (host) Consistency probe of the workspace layout: the kernels pad the K centroid rows up to
 * whole chunks of their own blocking (Section 3.2: several tile shapes per problem), and the
 * prologue writes -||c||^2/2 for every padded row.  Reports the largest padded row count over
 * every kernel variant and fault-tolerance mode that can be dispatched or forced for the problem,
 * and the rows the workspace reserves; planned_max <= reserved must hold. */
ftk_status ftk_plan_padded_rows(ftk_dtype dtype, int64_t N, int32_t D, int32_t K,
                                int64_t *planned_max /* (host) */, int64_t *reserved /* (host) */);

/* Assignment step, Eq. (1), Sections 3.1.2-3.1.5 and 4.
 *   X [N x D], C [K x D]  in  : read only.
 *   labels [N] int32      out : index of the nearest centroid.
 *   mindist [N] (dtype)   out : squared distance to it, >= 0; may be NULL.  Accuracy: points whose
 *                               decision was settled by exact re-evaluation, and every point of
 *                               the register-resident fp32 kernels (D <= 32; 32 < D <= 128 where
 *                               that kernel is dispatched), get the direct-difference value
 *                               (relative error of a few units in the last place of the
 *                               distance).  Otherwise the value comes from the expanded form of
 *                               Section 3.1.2, whose cancellation leaves an ABSOLUTE error of up
 *                               to 1.5 * band_coef * (||x_i|| max||c|| + max||c||^2/2) with
 *                               band_coef from ftk_ft_thresholds - small against the distance
 *                               unless the data sit far from the origin.
 *   faults [n_faults]     in  : soft errors to inject; NULL / 0 for none.  Ignored when
 *                               ft == FTK_FT_OFF is combined with n_faults == 0 only; with
 *                               FT off, listed faults are still injected (and corrupt the
 *                               result) so that the unprotected baseline can be observed.
 *   stats                 i/o : counters, may be NULL.
 * Requires 1 <= N, 1 <= D, 1 <= K, N*D < 2^40. */
ftk_status ftk_kmeans_assign(ftk_dtype dtype, const void *X, const void *C, int64_t N, int32_t D,
                             int32_t K, int32_t *labels, void *mindist, ftk_ft_mode ft,
                             const ftk_fault *faults, int32_t n_faults, ftk_ft_stats *stats,
                             void *workspace, size_t workspace_bytes, void *hip_stream);

/* ftk_kmeans_assign for callers that cannot allocate device memory or size a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * kernels and results as ftk_kmeans_assign, but the scratch (half norms, checksum rows, the
 * refine work-list and its counters) lives in a static device array inside the library:
 * ftk_static_scratch_bytes() = 16 MiB per GPU the library runs on, held until the process ends.
 * The call allocates nothing (no hipMalloc / hipFree, no events; the profiling aid below does
 * not apply to it).  A problem whose scratch exceeds the array (roughly N > 4 million points, or
 * K*D beyond a few million) is rejected with FTK_EWORKSPACE and nothing is enqueued.  Every call
 * on a GPU shares that GPU's array: calls must be ordered on one stream; calls that overlap on
 * one GPU race.  The buffer keeps the last call's contents; everything that must start at zero
 * is cleared by the call itself. */
size_t ftk_static_scratch_bytes(void);
ftk_status ftk_kmeans_assign_static(ftk_dtype dtype, const void *X, const void *C, int64_t N, int32_t D,
                                    int32_t K, int32_t *labels, void *mindist /* nullable */,
                                    ftk_ft_mode ft, const ftk_fault *faults, int32_t n_faults,
                                    ftk_ft_stats *stats /* nullable */, void *hip_stream);

/* Assignment step on the reduced-precision matrix path - the counterpart of the paper's TF32
 * tensor-core variant (Section 3.1.5; gfx950 has no TF32 format, its fast matrix format is bf16).
 * Same outputs and tie rule as ftk_kmeans_assign with fault tolerance off.  fp32 operands are
 * split into bf16 pieces and the piece products are accumulated in fp32 by the bf16 matrix
 * instructions: three pieces each and the six largest products for D <= 32, two pieces each and
 * all four products for 32 < D <= 128 (the wider rows' instruction count makes the certified
 * bound of the three-piece form nearly as wide, see ftk_fast_plan's band_coef).  The error bound
 * of that evaluation is known, and points whose best scores fall inside it are settled by exact
 * re-evaluation as in the fp32 path, so labels meet the same tolerance (identical to the exact
 * arg-min except on near-exact ties) and mindist is the exact-form distance to the chosen
 * centroid.
 * Covers dtype == FTK_F32 with D <= 128 and D a multiple of 4, X and C 16-byte aligned; anything
 * else returns FTK_EINVAL / FTK_EALIGN.
 * ft, faults, stats as for ftk_kmeans_assign: the paper protects its tensor-core variant with the
 * same checksums as the fp32 one (Sections 3.1.5 and 4), and so does this path - tiles of 30
 * centroids whose two checksum rows are split into bf16 pieces like any centroid row and go
 * through the same matrix instructions as the scores they must equal; detection, location,
 * correction, strict mode, the detection threshold (ftk_fast_plan reports it) and the injection
 * hook are those of the register-resident fp32 kernels.
 * workspace: ftk_workspace_bytes(dtype, N, D, K, ft) bytes. */
ftk_status ftk_kmeans_assign_fast(ftk_dtype dtype, const void *X, const void *C, int64_t N, int32_t D,
                                  int32_t K, int32_t *labels, void *mindist /* nullable */,
                                  ftk_ft_mode ft, const ftk_fault *faults /* nullable */, int32_t n_faults,
                                  ftk_ft_stats *stats /* nullable */, void *workspace, size_t workspace_bytes,
                                  void *hip_stream);

/* (host) What ftk_assign_geometry and ftk_ft_thresholds report, for the reduced-precision path:
 * the extents fault descriptors are taken modulo, the detection threshold and the settlement band
 * (both as multiples of B_i, see ftk_ft_thresholds).  For 32 < D <= 128 detect_coef is an upper
 * bound: the kernel's threshold is the rounding term plus ||x_i|| times the measured truncation
 * of the two-piece checksum rows, which is at most (and typically a tenth of) the 2^-16 * 15 *
 * max||c|| counted here.  Any output may be NULL. */
ftk_status ftk_fast_plan(ftk_dtype dtype, int64_t N, int32_t D, int32_t K, ftk_ft_mode ft,
                         ftk_geometry *geometry, double *detect_coef, double *band_coef);

/* Largest finite |x| over `count` elements, written as one double to out_absmax (device); NaN and
 * Inf elements are skipped.  ftk_kmeans_update needs it to fix the scale of its
 * order-independent accumulation. */
ftk_status ftk_absmax(ftk_dtype dtype, const void *X, int64_t count, double *out_absmax,
                      void *hip_stream);

/* Update step, Eq. (2), Sections 3.1.1-3.1.2 (sum the points of each cluster, then average).
 *   X [N x D], labels [N] in  : labels must lie in [0, K).
 *   C [K x D]             i/o : previous centroids in, new centroids out; rows of empty
 *                               clusters are left untouched.
 *   counts [K] int32      out : points per cluster.
 *   x_absmax              in  : device scalar from ftk_absmax over X, or NULL to have it
 *                               computed here (one more pass over X).
 * The result is bitwise reproducible from run to run: sums are accumulated in 64-bit fixed
 * point, which does not depend on the order of additions.
 * Accuracy: every coordinate is quantised once to a multiple of q = x_absmax * 2^-(61 - ceil(log2 N))
 * (fp32; at least 2^-50 x_absmax) or x_absmax * 2^-50 (fp64) before it is added, so a centroid
 * coordinate is off by at most q / 2 plus the final rounding to dtype, whatever its own
 * magnitude: one scale serves all features, and a feature whose values are many orders of
 * magnitude below the largest |x| of X keeps correspondingly fewer significant bits (for fp32
 * data and N = 2^20 the full 24 bits down to 2^-17 of the largest; for fp64 a feature 10^6
 * times smaller than the largest keeps about 31 bits).
 * X must be finite.  A NaN or Inf coordinate makes the centroid of the cluster its point is
 * labelled with unspecified (and, in the assignment, gives that point label 0 or any label in
 * range); all other clusters and points are unaffected, and nothing faults. */
ftk_status ftk_kmeans_update(ftk_dtype dtype, const void *X, const int32_t *labels, int64_t N,
                             int32_t D, int32_t K, void *C, int32_t *counts,
                             const double *x_absmax, void *workspace, size_t workspace_bytes,
                             void *hip_stream);

/* One Lloyd iteration (assignment, then update) carried out batch by batch: the single-pass idea of
 * Section 2.2 in the form this hardware allows.  The rows of X are taken in batches of `batch_rows`
 * points; each batch is assigned and, while it is still in the memory-side cache, added to the
 * running fixed-point sums; the centroids are averaged once after the last batch.  X is then read
 * from HBM once per iteration instead of twice, at the price of several launches per batch and of
 * a thinner grid per launch.  Results: labels and mindist as from ftk_kmeans_assign against the
 * incoming C; C and counts as from ftk_kmeans_update within its stated accuracy (the update always
 * runs on the per-workgroup table path here, so the last bits may differ from ftk_kmeans_update's).
 *   C [K x D]            i/o : centroids in, updated centroids out.
 *   x_absmax             in  : device scalar from ftk_absmax over X (required).
 *   batch_rows               : points per batch, at least N / 4096.
 * No fault tolerance on this path.  workspace: ftk_workspace_bytes(dtype, N, D, K, FTK_FT_OFF). */
ftk_status ftk_kmeans_step_batched(ftk_dtype dtype, const void *X, int64_t N, int32_t D, int32_t K, void *C,
                                   int32_t *labels, void *mindist /* nullable */, int32_t *counts,
                                   const double *x_absmax, int64_t batch_rows, void *workspace,
                                   size_t workspace_bytes, void *hip_stream);

/* The same update step protected by dual modular redundancy (Sections 2.3 and 4: the
 * memory-bound update is covered by duplicating its arithmetic and comparing).  With
 * ft != FTK_FT_OFF every arithmetic result of the step - conversion to fixed point, running
 * sums, member counts, table sums, scaling and division - is produced twice from the same
 * loaded operands and the two results are compared as integers before they leave the
 * registers (label-sorted path) or through a shadow total per workgroup (LDS-table path).
 *   DETECT           : a mismatch is counted (`detected`); the first result is used.
 *   CORRECT / STRICT : the affected run / workgroup pass is recomputed (`recomputed`; a pass
 *                      that mismatches again counts as `uncorrectable`), so the result equals
 *                      the fault-free one bit for bit.
 *   faults [n_faults] in : soft errors to inject into the first instruction stream of the
 *                      accumulating kernel: flip `bit` (mod 64) of the running sum / converted
 *                      operand number `reg` of lane `lane`, wave `wave`, workgroup `workgroup`,
 *                      after step `tile` of its row loop; extents from ftk_update_geometry.
 *                      With ft == FTK_FT_OFF they are injected unprotected.
 *   stats             i/o : injected / detected / recomputed / uncorrectable are added to. */
ftk_status ftk_kmeans_update_ft(ftk_dtype dtype, const void *X, const int32_t *labels, int64_t N,
                                int32_t D, int32_t K, void *C, int32_t *counts,
                                const double *x_absmax, ftk_ft_mode ft, const ftk_fault *faults,
                                int32_t n_faults, ftk_ft_stats *stats, void *workspace,
                                size_t workspace_bytes, void *hip_stream);

/* Extents of the fault coordinates of ftk_kmeans_update_ft (rows_aligned16: whether X rows are
 * 16-byte aligned, i.e. X % 16 == 0 and D * element size % 16 == 0). */
ftk_status ftk_update_geometry(ftk_dtype dtype, int64_t N, int32_t D, int32_t K,
                               int32_t rows_aligned16, ftk_geometry *out /* (host) */);

/* Lloyd loop, Section 2: `iters` times { assign ; update }, fixed iteration count.
 *   C_init [K x D]        in  : initial centroids, or NULL to take K distinct points of X
 *                               chosen by Floyd sampling driven by SplitMix64(seed)
 *                               (requires K <= N).
 *   C_out [K x D]         out : centroids after the last update.
 *   labels_out [N]        out : labels of the last assignment (taken against the centroids
 *                               before the last update).
 *   counts_out [K]        out : cluster sizes of that assignment.
 *   inertia_per_iter      out : (host, may be NULL) sum of mindist of every iteration;
 *                               when given, the call waits for the stream before returning.
 *   ft                        : mode of the assignment (checksums) and of the update (DMR).
 *   stats                 i/o : fault-tolerance counters summed over iterations, may be NULL. */
ftk_status ftk_kmeans_fit(ftk_dtype dtype, const void *X, int64_t N, int32_t D, int32_t K,
                          int32_t iters, uint64_t seed, const void *C_init, void *C_out,
                          int32_t *labels_out, int32_t *counts_out, double *inertia_per_iter,
                          ftk_ft_mode ft, ftk_ft_stats *stats, void *workspace,
                          size_t workspace_bytes, void *hip_stream);

/* The same loop with the assignment on the split-bf16 matrix path (ftk_kmeans_assign_fast):
 * fp32 data with D <= 128, D a multiple of 4, X 16-byte aligned.  Arguments as for
 * ftk_kmeans_fit, fault-tolerance mode (checksummed assignment, DMR update) and counters
 * included; workspace of ftk_workspace_bytes(dtype, N, D, K, ft) bytes. */
ftk_status ftk_kmeans_fit_fast(ftk_dtype dtype, const void *X, int64_t N, int32_t D, int32_t K,
                               int32_t iters, uint64_t seed, const void *C_init /* nullable */,
                               void *C_out, int32_t *labels_out, int32_t *counts_out,
                               double *inertia_per_iter /* (host) nullable */, ftk_ft_mode ft,
                               ftk_ft_stats *stats /* nullable */, void *workspace, size_t workspace_bytes,
                               void *hip_stream);

/* (host) K distinct indices in [0, N) by the seeded procedure ftk_kmeans_fit uses. */
ftk_status ftk_seeded_indices(uint64_t seed, int64_t N, int32_t K, int64_t *idx_host);

/* Profiling aid for benchmarks.  While enabled, every ftk_kmeans_assign call brackets its main
 * contraction kernel (not the small norm / refine kernels around it) with a pair of HIP events
 * recorded on the call's stream.  ftk_profile_read waits for all recorded pairs, returns the
 * summed kernel time in milliseconds and the number of launches since the last read (host
 * pointers), and releases the events.  Not thread-safe; creates events, so keep it out of
 * throughput timing loops. */
ftk_status ftk_profile_enable(int32_t on);
ftk_status ftk_profile_read(double *total_ms, int64_t *launches);

/* Hook for the shape-sweep / tuning tool (the counterpart of the paper's kernel selection,
 * Section 3.2: measure the candidates per problem shape, keep the fastest).  Forces, for every
 * later call of this process, the choices the library otherwise makes by rule; -1 restores a
 * rule.  Every forced choice computes the same results.
 *   assign_variant : 0 = generic kernel, 1 = the register-resident kernels where they apply
 *                    (fp32, 16-byte aligned rows: the small-D kernel for D <= 32, the mid-D
 *                    kernel for 32 < D <= 128 with D a multiple of 4)
 *   generic_tiles  : centroid tiles per chunk of the generic kernel, 1, 2, 4 or 8 (8: one point
 *                    tile per wave instead of two; chosen by rule only for fp64 with long rows)
 *   update_path    : 0 = per-workgroup LDS tables, 1 = label-sorted gather
 * Process-wide and not synchronised: set it while no call is in flight.  The workspace size
 * does not depend on it. */
ftk_status ftk_tuning_override(int32_t assign_variant, int32_t generic_tiles, int32_t update_path);

const char *ftk_last_error(void);
const char *ftk_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FTKMEANS_H */
