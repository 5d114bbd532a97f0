// Internal declarations shared by the translation units of libftkmeans (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ftkmeans.h"

namespace ftk {

// ---- error reporting -------------------------------------------------------------------
void set_error(const char *fmt, ...) __attribute__((format(printf, 1, 2)));
ftk_status hip_failed(hipError_t e, const char *what);

#define FTK_TRY_HIP(expr)                                      \
    do {                                                       \
        hipError_t e_ = (expr);                                \
        if (e_ != hipSuccess) return ftk::hip_failed(e_, #expr); \
    } while (0)

#define FTK_TRY(expr)                  \
    do {                               \
        ftk_status s_ = (expr);        \
        if (s_ != FTK_OK) return s_;   \
    } while (0)

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---- kernel-selection overrides (ftk_tuning_override; -1 = built-in rule) ------------------
struct Tuning {
    int assign_variant;  // 0 generic, 1 register-resident (small-D / mid-D) where it applies
    int kt;              // centroid tiles per chunk of the generic kernel: 1, 2 or 4
    int update_path;     // 0 LDS tables, 1 label-sorted
};
extern Tuning g_tuning;

// ---- assignment kernel geometry ----------------------------------------------------------
// One output tile of the matrix instruction covers TM centroids (rows, register axis) by TN
// points (columns, lane axis).  A wave owns PT point tiles and keeps KT centroid tiles of
// accumulators per point tile; a workgroup has 4 waves.
enum AssignVariant : int {
    VAR_GENERIC = 0,  // any D, any K: K in chunks of KT tiles, D streamed through LDS
    VAR_SMALLD = 1,   // fp32, D <= 32: point fragments stay in registers for the whole sweep
    VAR_MIDD = 2      // fp32, 32 < D <= 128: the same blocking, centroids LDS-resident, scores of the best tile kept
};

struct AssignPlan {
    AssignVariant variant;
    int TM, TN, PT, KT, waves;  // tile extents and per-wave blocking
    int KC;                     // centroids per K-chunk (= KT*TM)
    int nkc;                    // number of K-chunks
    int D8;                     // D rounded up to a multiple of 8
    int DQ;                     // quads (8 features) per LDS stage
    int points_per_wg;
    int64_t workgroups;
    int tiles_per_wave;         // output tiles a wave finishes (fault addressing)
    int regs_per_tile;
    size_t lds_bytes;
    bool hcn_pad_inf;           // padding rows of the half-norm vector hold +inf (never win)
    int grid;                   // workgroups launched (persistent variants launch fewer)
    int kch;                    // centroids staged in LDS at a time (small-D variant)
    double ft_coef;             // checksum detection threshold = ft_coef * (||x|| max||c|| + max||c||^2/2)
    double band_coef;           // rounding band of a score comparison, same scale
    double ft_trunc_coef;       // upper bound of what the kernel adds to ft_coef for truncated checksum rows (else 0)
};
AssignPlan plan_assign(ftk_dtype dtype, int64_t N, int D, int K, ftk_ft_mode ft, bool aligned16);

// ---- workspace carving --------------------------------------------------------------------
struct Workspace {
    // assignment
    void *hcn;          // [Kpad] half squared centroid norms (dtype), zero padded
    size_t hcn_entries; // Kpad: entries reserved for hcn
    double *scal;       // [8]   0: max_j ||c_j||^2 (as double bits, atomically maximised);
                        //       1: max truncation norm of a checksum row (two-piece fast path, same encoding)
    void *chk_v1;       // [nkc*KT][D8] per-tile plain checksum rows (dtype)
    void *chk_v2;       // [nkc*KT][D8] per-tile weighted checksum rows (dtype)
    void *chk_s;        // [nkc*KT][2]  their half-norm terms (dtype; small-D variant)
    double *chk_sd;     // [nkc][2]     the same per K-chunk, in double (generic variant)
    int32_t *wl_count;  // [4]   0: refine work-list length, 1: block counter (small-D / fast kernels)
    int32_t *wl;        // [N]   refine work-list (point indices)
    int32_t *wg_refined;  // [N/64 + 2] points each workgroup of the generic kernel settled in place
    // update
    int64_t *fx_sums;   // [K*D][2] fixed-point sums, two limbs (label-sorted path)
    int64_t *upd_slab;  // [chunks][K*D] per-workgroup fixed-point tables (LDS path), or
                        // [walkers][2][D] tagged partial sums (label-sorted path)
    int32_t *upd_cslab; // [chunks][K] per-workgroup member counts, or [walkers][2] slot tags
    double *absmax;     // [2]
    int32_t *sort_idx;  // [N]   point indices grouped by label
    int32_t *sort_lab;  // [N]   their labels
    int32_t *sort_cursor;  // [K+1] segment starts, after the scatter segment ends; [K] = total
    // fit
    void *C_cur;        // [K*D] running centroids (dtype)
    void *mindist;      // [N]   (dtype)
    double *inertia;    // [iters_max] per-iteration objective
    double *partials;   // [1024] block partial sums
    int64_t *idx;       // [K]   seeded initial point indices
    // fast (split-bf16) assignment
    void *csplit;       // centroid pieces in LDS image order (fp32 data with D <= 128, else empty)
    int32_t *batch_counters;  // [4 * MAX_BATCHES] work-list counters per batch of the batched step
    size_t total;
};
constexpr int FIT_MAX_ITERS_IN_WS = 4096;
constexpr int MAX_BATCHES = 4096;
size_t hcn_entries_max(ftk_dtype dtype, int64_t N, int D, int K);
// assign_only: stop after the assignment step's buffers (a prefix of the full layout)
Workspace carve_workspace(void *base, ftk_dtype dtype, int64_t N, int D, int K, ftk_ft_mode ft,
                          bool assign_only = false);
// upper bounds of the update step's per-workgroup tables, independent of pointer alignment
int64_t update_slab_chunks_max(int64_t N);
int64_t update_slab_cells_max(int64_t N, int D, int K);
int64_t update_walkers_max(int64_t N);

// ---- launches (each returns after enqueueing on `st`) ------------------------------------
struct AssignCall {
    ftk_dtype dtype;
    const void *X, *C;
    int64_t N;
    int D, K;
    int32_t *labels;
    void *mindist;
    ftk_ft_mode ft;
    const ftk_fault *faults;
    int n_faults;
    ftk_ft_stats *stats;
};
ftk_status launch_centroid_prologue(const AssignCall &c, const AssignPlan &p, const Workspace &w,
                                    hipStream_t st);
ftk_status launch_smalld_checksums(const AssignCall &c, const AssignPlan &p, const Workspace &w,
                                   hipStream_t st);
ftk_status launch_assign(const AssignCall &c, const AssignPlan &p, const Workspace &w, hipStream_t st);
// n_wg: workgroups of the preceding main kernel that left a settled-in-place count (generic
// kernel with statistics requested), else 0
ftk_status launch_refine(const AssignCall &c, const Workspace &w, int n_wg, hipStream_t st);
bool fast_supported(ftk_dtype dtype, int D);
size_t fast_split_bytes(ftk_dtype dtype, int D, int K);
void plan_fast(int64_t N, int D, int K, ftk_ft_mode ft, AssignPlan &p);
ftk_status launch_assign_fast(const AssignCall &c, const AssignPlan &p, const Workspace &w, hipStream_t st);

ftk_status launch_absmax(ftk_dtype dtype, const void *X, int64_t count, double *out, hipStream_t st);
ftk_status launch_update(ftk_dtype dtype, const void *X, const int32_t *labels, int64_t N, int D,
                         int K, void *C, int32_t *counts, const double *absmax, const Workspace &w,
                         ftk_ft_mode ft_mode, const ftk_fault *faults, int n_faults, ftk_ft_stats *stats,
                         hipStream_t st);
// update accumulated over several launches (batches of rows), finished by one averaging pass
struct BatchedUpdatePlan {
    int Ks, Ds, nks, nds, tx_log2, chunks;
    bool aligned, ok;
    int64_t scale_rows;
};
BatchedUpdatePlan plan_update_batched(ftk_dtype dtype, const void *X, int64_t N, int64_t batch_rows, int D, int K);
ftk_status launch_update_batch(ftk_dtype dtype, const void *Xb, const int32_t *labels_b, int64_t nb, int D, int K,
                               const double *absmax, const Workspace &w, const BatchedUpdatePlan &b, bool first,
                               hipStream_t st);
ftk_status launch_update_batched_finalize(ftk_dtype dtype, int D, int K, const double *absmax, void *C,
                                          int32_t *counts, const Workspace &w, const BatchedUpdatePlan &b,
                                          hipStream_t st);
ftk_status launch_zero_ints(int32_t *p, int n, hipStream_t st);
void update_geometry(ftk_dtype dtype, bool aligned16, int64_t N, int D, int K, ftk_geometry *out);
ftk_status launch_gather_rows(ftk_dtype dtype, const void *X, int D, const int64_t *idx_dev, int K,
                              void *C, hipStream_t st);
ftk_status launch_sum_to_double(ftk_dtype dtype, const void *v, int64_t n, double *partials,
                                double *out, hipStream_t st);

}  // namespace ftk
