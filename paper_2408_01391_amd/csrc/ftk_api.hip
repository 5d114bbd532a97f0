// C-ABI entry points of libftkmeans: argument checks, planning, workspace carving, and the
// host-side Lloyd loop (Section 2).  Everything numerical happens in the kernels.
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <unordered_set>
#include <utility>
#include <vector>

#include "ftk_internal.h"

namespace ftk {

static thread_local char g_err[512] = "";
Tuning g_tuning = {-1, -1, -1};

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

ftk_status hip_failed(hipError_t e, const char *what)
{
    set_error("HIP error %d (%s) in %s", (int)e, hipGetErrorString(e), what);
    return FTK_EDEVICE;
}

void plan_generic(ftk_dtype dtype, int64_t N, int D, int K, AssignPlan &p);
void plan_smalld(int64_t N, int D, int K, ftk_ft_mode ft, AssignPlan &p);
bool smalld_supported(ftk_dtype dtype, int D, int K);
void plan_midd(int64_t N, int D, int K, ftk_ft_mode ft, AssignPlan &p);
bool midd_supported(ftk_dtype dtype, int D, int K);
ftk_status launch_assign_midd(const AssignCall &c, const AssignPlan &p, const Workspace &w, hipStream_t st);
ftk_status launch_assign_generic(const AssignCall &c, const AssignPlan &p, const Workspace &w,
                                 hipStream_t st);
ftk_status launch_assign_smalld(const AssignCall &c, const AssignPlan &p, const Workspace &w,
                                hipStream_t st);

AssignPlan plan_assign(ftk_dtype dtype, int64_t N, int D, int K, ftk_ft_mode ft, bool aligned16)
{
    AssignPlan p;
    memset(&p, 0, sizeof(p));
    // The small-D kernel keeps the point fragments in registers and wins wherever there are enough
    // centroids to sweep; with few of them (K <= 128) and rows beyond 8 features the generic kernel
    // with its one- and two-tile blockings is faster (measured with the shape sweep's --tune: e.g.
    // D = 32, K = 32: 52 against 85 us for 2^20 points).
    bool few_centroids = D > 8 && (K <= 128 || (D >= 28 && K <= 256));
    if (ft != FTK_FT_OFF && smalld_supported(dtype, D, K)) {
        // With checksums the small-D kernel pays for its 30-centroid tiles, the per-tile verification
        // and (strict mode) the second sweep, the generic kernel for one vector-unit checksum per 128
        // centroids.  Measured at 2^20 points (whole call, CORRECT / STRICT): D = 32, K = 256: 196 against
        // 296 us for the generic kernel; D = 16, K = 256: 126 against 149; D = 32, K = 1024 - where the
        // checksummed tiles no longer fit LDS at once - 703 against 860; the small-D kernel keeps its
        // lead for D <= 12, for K >= 512 while its tiles stay resident, and from K = 4096 on.
        AssignPlan q;
        memset(&q, 0, sizeof(q));
        plan_smalld(N, D, K, ft, q);
        few_centroids = few_centroids || (D >= 16 && K <= 384) || (D >= 24 && K <= 512) ||
                        (D >= 24 && q.nkc > 1 && K <= 2048);
    }
    const bool want_smalld = g_tuning.assign_variant == 1 || (g_tuning.assign_variant == -1 && !few_centroids);
    // The mid-D kernel (rows of 33..128 features in registers, centroids in LDS) works in blocks of
    // 512 points, one workgroup per compute unit: it needs 2^17 points.  Measured against the
    // generic kernel at 2^17..2^20 points (A/B in one process).  Where the generic kernel runs its
    // condition-free stage loop (D a multiple of 16, K a multiple of 128) the mid-D kernel is 4-8 %
    // faster for D <= 64 from 256 centroids and for D <= 96 from 1024, equal or slower elsewhere,
    // and never faster with checksums (its tiles hold 30 centroids; the generic kernel verifies 128
    // at a time on the vector units at a third of the cost).  Against the guarded stage loop
    // (ragged D or K) it leads by 7-18 % for D <= 96 from 64 centroids on and by 6-7 % for wider
    // rows from 1024 on; with checksums for D <= 64 from 512 centroids, D <= 96 from 1024, any
    // width from 4096, and only for rows that fill the compiled width.
    bool midd_rule = false;
    if (N >= 131072) {
        const bool generic_whole = D % 16 == 0 && K % 128 == 0;
        if (ft == FTK_FT_OFF) {
            midd_rule = generic_whole ? ((D <= 64 && K >= 256) || (D <= 96 && K >= 1024))
                                      : ((D <= 96 && K >= 64) || K >= 1024);
        } else if (!generic_whole) {
            const int width = D <= 48 ? 48 : (D <= 64 ? 64 : (D <= 96 ? 96 : 128));
            midd_rule = 8 * D >= 7 * width && ((D <= 64 && K >= 512) || (D <= 96 && K >= 1024) || K >= 4096);
        }
    }
    const bool want_midd = g_tuning.assign_variant == 1 || (g_tuning.assign_variant == -1 && midd_rule);
    if (aligned16 && smalld_supported(dtype, D, K) && want_smalld)
        plan_smalld(N, D, K, ft, p);
    else if (aligned16 && midd_supported(dtype, D, K) && want_midd)
        plan_midd(N, D, K, ft, p);
    else
        plan_generic(dtype, N, D, K, p);
    return p;
}

ftk_status launch_assign(const AssignCall &c, const AssignPlan &p, const Workspace &w, hipStream_t st)
{
    if (p.variant == VAR_SMALLD) return launch_assign_smalld(c, p, w, st);
    if (p.variant == VAR_MIDD) return launch_assign_midd(c, p, w, st);
    return launch_assign_generic(c, p, w, st);
}

// Entries of the half-norm vector: every kernel variant pads K up to whole chunks of its own
// size (the small-D kernel to equal LDS chunks of 32-row tiles holding 30 or 32 centroids, the
// generic one to 1, 2, 4 or 8 tiles), and the prologue writes all of them.  The largest padding
// over all plans the dispatcher can choose, rounded up to 512, plus one block of slack.
size_t hcn_entries_max(ftk_dtype dtype, int64_t N, int D, int K)
{
    size_t need = (size_t)ceil_div(K, 128) * 128;  // generic: chunks of at most 128 centroids
    if (smalld_supported(dtype, D, K)) {
        for (ftk_ft_mode ft : {FTK_FT_OFF, FTK_FT_CORRECT, FTK_FT_STRICT}) {
            AssignPlan p;
            memset(&p, 0, sizeof(p));
            plan_smalld(N, D, K, ft, p);
            const size_t e = (size_t)p.nkc * p.KC;
            if (e > need) need = e;
        }
    }
    if (midd_supported(dtype, D, K)) {
        for (ftk_ft_mode ft : {FTK_FT_OFF, FTK_FT_CORRECT}) {
            AssignPlan p;
            memset(&p, 0, sizeof(p));
            plan_midd(N, D, K, ft, p);
            const size_t e = (size_t)p.nkc * p.KC;
            if (e > need) need = e;
        }
    }
    if (fast_supported(dtype, D)) {
        const size_t e = (size_t)ceil_div(K, 30) * 32;  // tiles of 30 centroids with checksums
        if (e > need) need = e;
    }
    return (size_t)ceil_div((int64_t)need, 512) * 512 + 512;
}

// The workspace is carved for the larger of the two kernel variants so that its size does not
// depend on which one the dispatcher picks.
Workspace carve_workspace(void *base, ftk_dtype dtype, int64_t N, int D, int K, ftk_ft_mode ft,
                          bool assign_only)
{
    (void)ft;
    const size_t esz = dtype == FTK_F32 ? 4 : 8;
    const size_t D8 = (size_t)ceil_div(D, 8) * 8;
    const size_t Kpad = hcn_entries_max(dtype, N, D, K);        // padded rows of the widest plan
    const size_t ntiles = Kpad / 8;                             // generous: checksum rows per lane group
    char *p = (char *)base;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        void *r = p ? (void *)(p + off) : nullptr;
        off += align_up(bytes, 256);
        return r;
    };
    Workspace w;
    w.hcn = take(Kpad * esz);
    w.hcn_entries = Kpad;
    w.scal = (double *)take(8 * sizeof(double));
    w.chk_v1 = take(ntiles * D8 * esz);
    w.chk_v2 = take(ntiles * D8 * esz);
    w.chk_s = take(ntiles * 2 * esz);
    w.chk_sd = (double *)take(ntiles * 2 * sizeof(double));
    w.wl_count = (int32_t *)take(4 * sizeof(int32_t));
    w.wl = (int32_t *)take((size_t)N * sizeof(int32_t));
    w.wg_refined = (int32_t *)take(((size_t)N / 64 + 2) * sizeof(int32_t));
    if (assign_only) {  // the assignment step touches nothing beyond this point
        w.fx_sums = nullptr;
        w.upd_slab = nullptr;
        w.upd_cslab = nullptr;
        w.absmax = nullptr;
        w.sort_idx = w.sort_lab = w.sort_cursor = nullptr;
        w.C_cur = w.mindist = nullptr;
        w.inertia = w.partials = nullptr;
        w.idx = nullptr;
        w.csplit = nullptr;
        w.batch_counters = nullptr;
        w.total = off;
        return w;
    }
    w.fx_sums = (int64_t *)take((size_t)K * D * 2 * sizeof(int64_t));  // two limbs per cell
    {   // shared by the two update paths: per-workgroup tables, or two tagged slots per walker
        const size_t slab_cells = (size_t)update_slab_cells_max(N, D, K);
        const size_t slot_cells = (size_t)update_walkers_max(N) * 2 * (size_t)D;
        w.upd_slab = (int64_t *)take((slab_cells > slot_cells ? slab_cells : slot_cells) * sizeof(int64_t));
        const size_t slab_counts = (size_t)update_slab_chunks_max(N) * K;
        const size_t slot_tags = (size_t)update_walkers_max(N) * 2;
        w.upd_cslab = (int32_t *)take((slab_counts > slot_tags ? slab_counts : slot_tags) * sizeof(int32_t));
    }
    w.absmax = (double *)take(2 * sizeof(double));
    w.sort_idx = (int32_t *)take((size_t)N * sizeof(int32_t));
    w.sort_lab = (int32_t *)take((size_t)N * sizeof(int32_t));
    w.sort_cursor = (int32_t *)take(((size_t)K + 1) * sizeof(int32_t));
    w.C_cur = take((size_t)K * D * esz);
    w.mindist = take((size_t)N * esz);
    w.inertia = (double *)take(FIT_MAX_ITERS_IN_WS * sizeof(double));
    w.partials = (double *)take(1024 * sizeof(double));
    w.idx = (int64_t *)take((size_t)K * sizeof(int64_t));
    w.csplit = take(fast_split_bytes(dtype, D, K));
    w.batch_counters = (int32_t *)take((size_t)4 * MAX_BATCHES * sizeof(int32_t));
    w.total = off;
    return w;
}

static ftk_status check_problem(ftk_dtype dtype, int64_t N, int D, int K, int ft)
{
    if (dtype != FTK_F32 && dtype != FTK_F64) {
        set_error("unknown dtype %d", (int)dtype);
        return FTK_EINVAL;
    }
    if (ft != FTK_FT_OFF && ft != FTK_FT_DETECT && ft != FTK_FT_CORRECT && ft != FTK_FT_STRICT) {
        set_error("unknown ft_mode %d", ft);
        return FTK_EINVAL;
    }
    if (N < 1 || D < 1 || K < 1) {
        set_error("need N >= 1, D >= 1, K >= 1 (got N=%lld D=%d K=%d)", (long long)N, D, K);
        return FTK_EINVAL;
    }
    if (N > 0x7fffffffLL || (double)N * D >= 1099511627776.0 || (int64_t)K * D > (1LL << 31)) {
        set_error("problem too large: N=%lld D=%d K=%d (need N < 2^31, N*D < 2^40, K*D <= 2^31)",
                  (long long)N, D, K);
        return FTK_EINVAL;
    }
    return FTK_OK;
}

static ftk_status check_ptr(const void *p, size_t align, const char *name)
{
    if (!p) {
        set_error("%s is NULL", name);
        return FTK_EINVAL;
    }
    if ((uintptr_t)p % align) {
        set_error("%s is not %zu-byte aligned", name, align);
        return FTK_EALIGN;
    }
    return FTK_OK;
}

static ftk_status check_workspace(void *ws, size_t bytes, size_t need)
{
    if (!ws || bytes < need) {
        set_error("workspace of %zu bytes given, %zu needed", ws ? bytes : (size_t)0, need);
        return FTK_EWORKSPACE;
    }
    if ((uintptr_t)ws % 256) {
        set_error("workspace is not 256-byte aligned");
        return FTK_EALIGN;
    }
    return FTK_OK;
}

static ftk_status check_device()
{
    static thread_local int checked_dev = -1;
    int dev = 0;
    FTK_TRY_HIP(hipGetDevice(&dev));
    if (dev == checked_dev) return FTK_OK;
    hipDeviceProp_t prop;
    FTK_TRY_HIP(hipGetDeviceProperties(&prop, dev));
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0) {
        set_error("device %d is %s; this library is built for gfx950 only", dev, prop.gcnArchName);
        return FTK_EDEVICE;
    }
    checked_dev = dev;
    return FTK_OK;
}

static bool g_profile = false;
static std::vector<std::pair<hipEvent_t, hipEvent_t>> g_profile_events;

static ftk_status assign_impl(const AssignCall &c, void *workspace, hipStream_t st, bool fast = false,
                              bool allow_profile = true)
{
    const bool aligned16 = ((uintptr_t)c.X % 16 == 0) && ((uintptr_t)c.C % 16 == 0);
    AssignPlan p;
    if (fast) {
        memset(&p, 0, sizeof(p));
        plan_fast(c.N, c.D, c.K, c.ft, p);
    } else {
        p = plan_assign(c.dtype, c.N, c.D, c.K, c.ft, aligned16);
    }
    // the carve is a prefix of the full one, so the assignment-only layout serves both callers
    const Workspace w = carve_workspace(workspace, c.dtype, c.N, c.D, c.K, c.ft, !fast);
    FTK_TRY(launch_centroid_prologue(c, p, w, st));
    hipEvent_t e0 = nullptr, e1 = nullptr;
    // at most 65536 pending pairs: a caller that enables profiling and never reads stops recording
    const bool profile = g_profile && allow_profile && g_profile_events.size() < 65536;
    if (profile) {
        FTK_TRY_HIP(hipEventCreate(&e0));
        if (hipError_t e = hipEventCreate(&e1); e != hipSuccess) {
            (void)hipEventDestroy(e0);
            return hip_failed(e, "hipEventCreate");
        }
        FTK_TRY_HIP(hipEventRecord(e0, st));
    }
    if (fast)
        FTK_TRY(launch_assign_fast(c, p, w, st));
    else
        FTK_TRY(launch_assign(c, p, w, st));
    if (profile) {
        g_profile_events.emplace_back(e0, e1);  // owned by the list from here on
        FTK_TRY_HIP(hipEventRecord(e1, st));
    }
    const int n_wg = (!fast && c.stats && p.variant == VAR_GENERIC) ? (int)p.workgroups : 0;
    FTK_TRY(launch_refine(c, w, n_wg, st));
    return FTK_OK;
}

}  // namespace ftk

// ---- scratch of the entry point that allocates nothing ------------------------------------
// One array per GPU, part of the loaded code object, held until the process ends.  In host code
// its name is only a handle: the device address is looked up once per device and that pointer is
// what the kernels get.
#define FTK_STATIC_SCRATCH_BYTES (16u << 20)
static __device__ __align__(256) unsigned char ftk_static_scratch[FTK_STATIC_SCRATCH_BYTES];

namespace ftk {
constexpr int STATIC_MAX_DEVICES = 64;
static std::mutex g_static_mutex;
static void *g_static_ptr[STATIC_MAX_DEVICES] = {};

static ftk_status static_scratch_of_current_device(void **out)
{
    int dev = 0;
    FTK_TRY_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= STATIC_MAX_DEVICES) {
        set_error("device ordinal %d beyond the %d this library keeps scratch for", dev, STATIC_MAX_DEVICES);
        return FTK_EDEVICE;
    }
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ptr[dev]) {
        void *ptr = nullptr;
        FTK_TRY_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(ftk_static_scratch)));
        if (!ptr || (uintptr_t)ptr % 256) {
            set_error("static scratch of device %d resolved to %p", dev, ptr);
            return FTK_EDEVICE;
        }
        g_static_ptr[dev] = ptr;
    }
    *out = g_static_ptr[dev];
    return FTK_OK;
}
}  // namespace ftk

using namespace ftk;

extern "C" {

ftk_status ftk_profile_enable(int32_t on)
{
    g_profile = on != 0;
    return FTK_OK;
}

ftk_status ftk_profile_read(double *total_ms, int64_t *launches)
{
    if (!total_ms || !launches) {
        set_error("NULL output");
        return FTK_EINVAL;
    }
    double sum = 0.0;
    int64_t n = 0;
    for (auto &pr : g_profile_events) {
        float ms = 0.f;
        FTK_TRY_HIP(hipEventSynchronize(pr.second));
        FTK_TRY_HIP(hipEventElapsedTime(&ms, pr.first, pr.second));
        sum += ms;
        ++n;
        (void)hipEventDestroy(pr.first);
        (void)hipEventDestroy(pr.second);
    }
    g_profile_events.clear();
    *total_ms = sum;
    *launches = n;
    return FTK_OK;
}

ftk_status ftk_tuning_override(int32_t assign_variant, int32_t generic_tiles, int32_t update_path)
{
    if (assign_variant < -1 || assign_variant > 1 || update_path < -1 || update_path > 1 ||
        !(generic_tiles == -1 || generic_tiles == 1 || generic_tiles == 2 || generic_tiles == 4 || generic_tiles == 8)) {
        set_error("tuning override out of range (%d, %d, %d)", assign_variant, generic_tiles, update_path);
        return FTK_EINVAL;
    }
    g_tuning = Tuning{assign_variant, generic_tiles, update_path};
    return FTK_OK;
}

const char *ftk_last_error(void) { return g_err; }
const char *ftk_version(void) { return "ftkmeans 0.1 (gfx950)"; }

size_t ftk_workspace_bytes(ftk_dtype dtype, int64_t N, int32_t D, int32_t K, ftk_ft_mode ft)
{
    if (check_problem(dtype, N, D, K, ft) != FTK_OK) return 0;
    return carve_workspace(nullptr, dtype, N, D, K, ft).total;
}

ftk_status ftk_assign_geometry(ftk_dtype dtype, int64_t N, int32_t D, int32_t K, ftk_ft_mode ft,
                               ftk_geometry *out)
{
    FTK_TRY(check_problem(dtype, N, D, K, ft));
    if (!out) {
        set_error("out is NULL");
        return FTK_EINVAL;
    }
    const AssignPlan p = plan_assign(dtype, N, D, K, ft, true);
    out->workgroups = (uint32_t)p.workgroups;
    out->waves_per_workgroup = (uint32_t)p.waves;
    out->tiles_per_wave = (uint32_t)p.tiles_per_wave;
    out->regs_per_tile = (uint32_t)p.regs_per_tile;
    out->lanes = 64;
    out->bits = dtype == FTK_F32 ? 32 : 64;
    return FTK_OK;
}

ftk_status ftk_ft_thresholds(ftk_dtype dtype, int64_t N, int32_t D, int32_t K, ftk_ft_mode ft,
                             double *detect_coef, double *band_coef)
{
    FTK_TRY(check_problem(dtype, N, D, K, ft));
    if (!detect_coef || !band_coef) {
        set_error("NULL output");
        return FTK_EINVAL;
    }
    const AssignPlan p = plan_assign(dtype, N, D, K, ft, true);
    *detect_coef = ft == FTK_FT_OFF ? 0.0 : p.ft_coef;
    *band_coef = p.band_coef;
    return FTK_OK;
}

ftk_status ftk_plan_padded_rows(ftk_dtype dtype, int64_t N, int32_t D, int32_t K, int64_t *planned_max,
                                int64_t *reserved)
{
    FTK_TRY(check_problem(dtype, N, D, K, FTK_FT_OFF));
    if (!planned_max || !reserved) {
        set_error("NULL output");
        return FTK_EINVAL;
    }
    // every plan the dispatcher or a tuning override can produce
    int64_t worst = 0;
    const Tuning saved = g_tuning;
    for (int variant = 0; variant <= 1; ++variant)
        for (int kt : {1, 2, 4, 8})
            for (ftk_ft_mode ft : {FTK_FT_OFF, FTK_FT_DETECT, FTK_FT_CORRECT, FTK_FT_STRICT}) {
                g_tuning = Tuning{variant, kt, -1};
                const AssignPlan p = plan_assign(dtype, N, D, K, ft, true);
                const int64_t rows = (int64_t)p.nkc * p.KC;
                if (rows > worst) worst = rows;
            }
    g_tuning = saved;
    if (fast_supported(dtype, D)) {
        for (ftk_ft_mode ft : {FTK_FT_OFF, FTK_FT_CORRECT}) {
            AssignPlan p;
            memset(&p, 0, sizeof(p));
            plan_fast(N, D, K, ft, p);
            const int64_t rows = (int64_t)p.nkc * p.KC;
            if (rows > worst) worst = rows;
        }
    }
    *planned_max = worst;
    *reserved = (int64_t)hcn_entries_max(dtype, N, D, K);
    return FTK_OK;
}

ftk_status ftk_kmeans_assign(ftk_dtype dtype, const void *X, const void *C, int64_t N, int32_t D,
                             int32_t K, int32_t *labels, void *mindist, ftk_ft_mode ft,
                             const ftk_fault *faults, int32_t n_faults, ftk_ft_stats *stats,
                             void *workspace, size_t workspace_bytes, void *hip_stream)
{
    FTK_TRY(check_problem(dtype, N, D, K, ft));
    const size_t esz = dtype == FTK_F32 ? 4 : 8;
    FTK_TRY(check_ptr(X, esz, "X"));
    FTK_TRY(check_ptr(C, esz, "C"));
    FTK_TRY(check_ptr(labels, 4, "labels"));
    if (mindist) FTK_TRY(check_ptr(mindist, esz, "mindist"));
    if (n_faults < 0 || (n_faults > 0 && !faults)) {
        set_error("n_faults=%d with faults=%p", n_faults, (const void *)faults);
        return FTK_EINVAL;
    }
    if (stats) FTK_TRY(check_ptr(stats, 8, "stats"));
    FTK_TRY(check_workspace(workspace, workspace_bytes, ftk_workspace_bytes(dtype, N, D, K, ft)));
    FTK_TRY(check_device());
    AssignCall c{dtype, X, C, N, D, K, labels, mindist, ft, faults, n_faults, stats};
    return assign_impl(c, workspace, (hipStream_t)hip_stream);
}

size_t ftk_static_scratch_bytes(void) { return FTK_STATIC_SCRATCH_BYTES; }

ftk_status ftk_kmeans_assign_static(ftk_dtype dtype, const void *X, const void *C, int64_t N, int32_t D,
                                    int32_t K, int32_t *labels, void *mindist, ftk_ft_mode ft,
                                    const ftk_fault *faults, int32_t n_faults, ftk_ft_stats *stats,
                                    void *hip_stream)
{
    FTK_TRY(check_problem(dtype, N, D, K, ft));
    const size_t esz = dtype == FTK_F32 ? 4 : 8;
    FTK_TRY(check_ptr(X, esz, "X"));
    FTK_TRY(check_ptr(C, esz, "C"));
    FTK_TRY(check_ptr(labels, 4, "labels"));
    if (mindist) FTK_TRY(check_ptr(mindist, esz, "mindist"));
    if (n_faults < 0 || (n_faults > 0 && !faults)) {
        set_error("n_faults=%d with faults=%p", n_faults, (const void *)faults);
        return FTK_EINVAL;
    }
    if (stats) FTK_TRY(check_ptr(stats, 8, "stats"));
    const size_t need = carve_workspace(nullptr, dtype, N, D, K, ft, true).total;
    if (need > FTK_STATIC_SCRATCH_BYTES) {
        set_error("problem needs %zu bytes of scratch, the static buffer holds %zu (N=%lld D=%d K=%d): "
                  "use ftk_kmeans_assign with a caller workspace", need, (size_t)FTK_STATIC_SCRATCH_BYTES,
                  (long long)N, D, K);
        return FTK_EWORKSPACE;
    }
    FTK_TRY(check_device());
    void *scratch = nullptr;
    FTK_TRY(static_scratch_of_current_device(&scratch));
    AssignCall c{dtype, X, C, N, D, K, labels, mindist, ft, faults, n_faults, stats};
    return assign_impl(c, scratch, (hipStream_t)hip_stream, false, false);
}

static ftk_status check_fast(ftk_dtype dtype, int D)
{
    if (!fast_supported(dtype, D)) {
        set_error("the fast assignment covers fp32 data with D <= 128 and D a multiple of 4 (got dtype=%d D=%d)",
                  (int)dtype, D);
        return FTK_EINVAL;
    }
    return FTK_OK;
}

ftk_status ftk_kmeans_assign_fast(ftk_dtype dtype, const void *X, const void *C, int64_t N, int32_t D,
                                  int32_t K, int32_t *labels, void *mindist, ftk_ft_mode ft,
                                  const ftk_fault *faults, int32_t n_faults, ftk_ft_stats *stats,
                                  void *workspace, size_t workspace_bytes, void *hip_stream)
{
    FTK_TRY(check_problem(dtype, N, D, K, ft));
    FTK_TRY(check_fast(dtype, D));
    FTK_TRY(check_ptr(X, 16, "X"));
    FTK_TRY(check_ptr(C, 16, "C"));
    FTK_TRY(check_ptr(labels, 4, "labels"));
    if (mindist) FTK_TRY(check_ptr(mindist, 4, "mindist"));
    if (stats) FTK_TRY(check_ptr(stats, 8, "stats"));
    if (n_faults < 0 || (n_faults > 0 && !faults)) {
        set_error("n_faults=%d with faults=%p", n_faults, (const void *)faults);
        return FTK_EINVAL;
    }
    FTK_TRY(check_workspace(workspace, workspace_bytes, ftk_workspace_bytes(dtype, N, D, K, ft)));
    FTK_TRY(check_device());
    AssignCall c{dtype, X, C, N, D, K, labels, mindist, ft, faults, n_faults, stats};
    return assign_impl(c, workspace, (hipStream_t)hip_stream, true);
}

ftk_status ftk_fast_plan(ftk_dtype dtype, int64_t N, int32_t D, int32_t K, ftk_ft_mode ft, ftk_geometry *geometry,
                         double *detect_coef, double *band_coef)
{
    FTK_TRY(check_problem(dtype, N, D, K, ft));
    FTK_TRY(check_fast(dtype, D));
    AssignPlan p;
    memset(&p, 0, sizeof(p));
    plan_fast(N, D, K, ft, p);
    if (geometry) {
        geometry->workgroups = (uint32_t)p.workgroups;
        geometry->waves_per_workgroup = (uint32_t)p.waves;
        geometry->tiles_per_wave = (uint32_t)p.tiles_per_wave;
        geometry->regs_per_tile = (uint32_t)p.regs_per_tile;
        geometry->lanes = 64;
        geometry->bits = 32;
    }
    if (detect_coef) *detect_coef = ft == FTK_FT_OFF ? 0.0 : p.ft_coef + p.ft_trunc_coef;
    if (band_coef) *band_coef = p.band_coef;
    return FTK_OK;
}

ftk_status ftk_absmax(ftk_dtype dtype, const void *X, int64_t count, double *out_absmax, void *hip_stream)
{
    if (dtype != FTK_F32 && dtype != FTK_F64) {
        set_error("unknown dtype %d", (int)dtype);
        return FTK_EINVAL;
    }
    if (count < 1) {
        set_error("count must be >= 1");
        return FTK_EINVAL;
    }
    FTK_TRY(check_ptr(X, dtype == FTK_F32 ? 4 : 8, "X"));
    FTK_TRY(check_ptr(out_absmax, 8, "out_absmax"));
    FTK_TRY(check_device());
    return launch_absmax(dtype, X, count, out_absmax, (hipStream_t)hip_stream);
}

ftk_status ftk_kmeans_update_ft(ftk_dtype dtype, const void *X, const int32_t *labels, int64_t N,
                                int32_t D, int32_t K, void *C, int32_t *counts, const double *x_absmax,
                                ftk_ft_mode ft, const ftk_fault *faults, int32_t n_faults,
                                ftk_ft_stats *stats, void *workspace, size_t workspace_bytes,
                                void *hip_stream)
{
    FTK_TRY(check_problem(dtype, N, D, K, ft));
    const size_t esz = dtype == FTK_F32 ? 4 : 8;
    FTK_TRY(check_ptr(X, esz, "X"));
    FTK_TRY(check_ptr(labels, 4, "labels"));
    FTK_TRY(check_ptr(C, esz, "C"));
    FTK_TRY(check_ptr(counts, 4, "counts"));
    if (x_absmax) FTK_TRY(check_ptr(x_absmax, 8, "x_absmax"));
    if (n_faults < 0 || (n_faults > 0 && !faults)) {
        set_error("n_faults = %d with faults = %p", n_faults, (const void *)faults);
        return FTK_EINVAL;
    }
    if (stats) FTK_TRY(check_ptr(stats, 8, "stats"));
    FTK_TRY(check_workspace(workspace, workspace_bytes, ftk_workspace_bytes(dtype, N, D, K, ft)));
    FTK_TRY(check_device());
    hipStream_t st = (hipStream_t)hip_stream;
    const Workspace w = carve_workspace(workspace, dtype, N, D, K, ft);
    if (!x_absmax) {
        FTK_TRY(launch_absmax(dtype, X, N * (int64_t)D, w.absmax, st));
        x_absmax = w.absmax;
    }
    return launch_update(dtype, X, labels, N, D, K, C, counts, x_absmax, w, ft, faults, n_faults, stats, st);
}

ftk_status ftk_kmeans_update(ftk_dtype dtype, const void *X, const int32_t *labels, int64_t N,
                             int32_t D, int32_t K, void *C, int32_t *counts, const double *x_absmax,
                             void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return ftk_kmeans_update_ft(dtype, X, labels, N, D, K, C, counts, x_absmax, FTK_FT_OFF, nullptr, 0,
                                nullptr, workspace, workspace_bytes, hip_stream);
}

ftk_status ftk_kmeans_step_batched(ftk_dtype dtype, const void *X, int64_t N, int32_t D, int32_t K, void *C,
                                   int32_t *labels, void *mindist, int32_t *counts, const double *x_absmax,
                                   int64_t batch_rows, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    FTK_TRY(check_problem(dtype, N, D, K, FTK_FT_OFF));
    const size_t esz = dtype == FTK_F32 ? 4 : 8;
    FTK_TRY(check_ptr(X, esz, "X"));
    FTK_TRY(check_ptr(C, esz, "C"));
    FTK_TRY(check_ptr(labels, 4, "labels"));
    if (mindist) FTK_TRY(check_ptr(mindist, esz, "mindist"));
    FTK_TRY(check_ptr(counts, 4, "counts"));
    FTK_TRY(check_ptr(x_absmax, 8, "x_absmax"));
    if (batch_rows < 1 || ceil_div(N, batch_rows) > MAX_BATCHES) {
        set_error("batch_rows = %lld gives %lld batches (allowed: 1 .. %d)", (long long)batch_rows,
                  batch_rows < 1 ? 0ll : (long long)ceil_div(N, batch_rows), MAX_BATCHES);
        return FTK_EINVAL;
    }
    FTK_TRY(check_workspace(workspace, workspace_bytes, ftk_workspace_bytes(dtype, N, D, K, FTK_FT_OFF)));
    FTK_TRY(check_device());
    hipStream_t st = (hipStream_t)hip_stream;
    const Workspace w = carve_workspace(workspace, dtype, N, D, K, FTK_FT_OFF);
    // whole rows of 16 bytes keep every batch as aligned as X itself
    const bool aligned16 = ((uintptr_t)X % 16 == 0) && ((uintptr_t)C % 16 == 0) && ((size_t)D * esz) % 16 == 0;
    const BatchedUpdatePlan ub = plan_update_batched(dtype, aligned16 ? X : (const void *)1, N, batch_rows, D, K);
    if (!ub.ok) {
        set_error("internal: update tables of a batch exceed the workspace bound (chunks %d)", ub.chunks);
        return FTK_EINVAL;
    }
    const int64_t nbatch = ceil_div(N, batch_rows);
    FTK_TRY(launch_zero_ints(w.batch_counters, (int)(4 * nbatch), st));
    // norms of the centroids once: they do not change inside the iteration
    AssignCall whole{dtype, X, C, batch_rows < N ? batch_rows : N, D, K, labels, mindist, FTK_FT_OFF, nullptr, 0, nullptr};
    AssignPlan pprev = plan_assign(dtype, whole.N, D, K, FTK_FT_OFF, aligned16);
    FTK_TRY(launch_centroid_prologue(whole, pprev, w, st));
    for (int64_t b = 0; b < nbatch; ++b) {
        const int64_t r0 = b * batch_rows;
        const int64_t nb = N - r0 < batch_rows ? N - r0 : batch_rows;
        const char *Xb = (const char *)X + (size_t)r0 * D * esz;
        AssignCall c{dtype, Xb, C, nb, D, K, labels + r0, mindist ? (void *)((char *)mindist + (size_t)r0 * esz) : nullptr,
                     FTK_FT_OFF, nullptr, 0, nullptr};
        AssignPlan p = plan_assign(dtype, nb, D, K, FTK_FT_OFF, aligned16);
        if (p.variant != pprev.variant || p.nkc * p.KC != pprev.nkc * pprev.KC || p.hcn_pad_inf != pprev.hcn_pad_inf) {
            // a shorter last batch may be planned for another kernel, whose padded norm vector differs
            FTK_TRY(launch_centroid_prologue(c, p, w, st));
            pprev = p;
        }
        Workspace wb = w;
        wb.wl_count = w.batch_counters + 4 * b;  // fresh work-list counters per batch
        FTK_TRY(launch_assign(c, p, wb, st));
        FTK_TRY(launch_refine(c, wb, 0, st));
        FTK_TRY(launch_update_batch(dtype, Xb, labels + r0, nb, D, K, x_absmax, w, ub, b == 0, st));
    }
    return launch_update_batched_finalize(dtype, D, K, x_absmax, C, counts, w, ub, st);
}

ftk_status ftk_update_geometry(ftk_dtype dtype, int64_t N, int32_t D, int32_t K, int32_t rows_aligned16,
                               ftk_geometry *out)
{
    FTK_TRY(check_problem(dtype, N, D, K, FTK_FT_OFF));
    if (!out) {
        set_error("out is NULL");
        return FTK_EINVAL;
    }
    update_geometry(dtype, rows_aligned16 != 0, N, D, K, out);
    return FTK_OK;
}

ftk_status ftk_seeded_indices(uint64_t seed, int64_t N, int32_t K, int64_t *idx_host)
{
    if (K < 1 || N < K || !idx_host) {
        set_error("need 1 <= K <= N and a destination (N=%lld K=%d)", (long long)N, K);
        return FTK_EINVAL;
    }
    // Floyd's sampling of K distinct values from [0, N), driven by SplitMix64.
    uint64_t state = seed;
    auto next = [&state]() {
        uint64_t z = (state += 0x9E3779B97F4A7C15ULL);
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
        return z ^ (z >> 31);
    };
    std::unordered_set<int64_t> chosen;
    chosen.reserve((size_t)K * 2);
    int filled = 0;
    for (int64_t top = N - K; top < N; ++top) {
        const int64_t pick = (int64_t)(next() % (uint64_t)(top + 1));
        const int64_t take = chosen.count(pick) ? top : pick;  // `top` itself cannot have been chosen yet
        chosen.insert(take);
        idx_host[filled++] = take;
    }
    return FTK_OK;
}

static ftk_status fit_impl(ftk_dtype dtype, const void *X, int64_t N, int32_t D, int32_t K,
                           int32_t iters, uint64_t seed, const void *C_init, void *C_out,
                           int32_t *labels_out, int32_t *counts_out, double *inertia_per_iter,
                           ftk_ft_mode ft, ftk_ft_stats *stats, void *workspace,
                           size_t workspace_bytes, void *hip_stream, bool fast)
{
    FTK_TRY(check_problem(dtype, N, D, K, ft));
    if (fast) {
        FTK_TRY(check_fast(dtype, D));
        FTK_TRY(check_ptr(X, 16, "X"));
    }
    if (iters < 0 || iters > FIT_MAX_ITERS_IN_WS) {
        set_error("iters must be in [0, %d]", FIT_MAX_ITERS_IN_WS);
        return FTK_EINVAL;
    }
    const size_t esz = dtype == FTK_F32 ? 4 : 8;
    FTK_TRY(check_ptr(X, esz, "X"));
    if (C_init) FTK_TRY(check_ptr(C_init, esz, "C_init"));
    FTK_TRY(check_ptr(C_out, esz, "C_out"));
    FTK_TRY(check_ptr(labels_out, 4, "labels_out"));
    FTK_TRY(check_ptr(counts_out, 4, "counts_out"));
    if (stats) FTK_TRY(check_ptr(stats, 8, "stats"));
    if (!C_init && K > N) {
        set_error("seeded initialisation needs K <= N (N=%lld K=%d)", (long long)N, K);
        return FTK_EINVAL;
    }
    FTK_TRY(check_workspace(workspace, workspace_bytes, ftk_workspace_bytes(dtype, N, D, K, ft)));
    FTK_TRY(check_device());
    hipStream_t st = (hipStream_t)hip_stream;
    const Workspace w = carve_workspace(workspace, dtype, N, D, K, ft);

    if (C_init) {
        FTK_TRY_HIP(hipMemcpyAsync(w.C_cur, C_init, (size_t)K * D * esz, hipMemcpyDeviceToDevice, st));
    } else {
        std::vector<int64_t> idx((size_t)K);
        FTK_TRY(ftk_seeded_indices(seed, N, K, idx.data()));
        FTK_TRY_HIP(hipMemcpyAsync(w.idx, idx.data(), (size_t)K * sizeof(int64_t), hipMemcpyHostToDevice, st));
        FTK_TRY_HIP(hipStreamSynchronize(st));  // idx lives on this stack frame
        FTK_TRY(launch_gather_rows(dtype, X, D, w.idx, K, w.C_cur, st));
    }
    FTK_TRY(launch_absmax(dtype, X, N * (int64_t)D, w.absmax, st));
    for (int t = 0; t < iters; ++t) {
        AssignCall c{dtype, X, w.C_cur, N, D, K, labels_out, w.mindist, ft, nullptr, 0, stats};
        FTK_TRY(assign_impl(c, workspace, st, fast));
        if (inertia_per_iter)
            FTK_TRY(launch_sum_to_double(dtype, w.mindist, N, w.partials, w.inertia + t, st));
        FTK_TRY(launch_update(dtype, X, labels_out, N, D, K, w.C_cur, counts_out, w.absmax, w, ft, nullptr, 0,
                              stats, st));
    }
    FTK_TRY_HIP(hipMemcpyAsync(C_out, w.C_cur, (size_t)K * D * esz, hipMemcpyDeviceToDevice, st));
    if (inertia_per_iter && iters > 0) {
        FTK_TRY_HIP(hipMemcpyAsync(inertia_per_iter, w.inertia, (size_t)iters * sizeof(double),
                                   hipMemcpyDeviceToHost, st));
        FTK_TRY_HIP(hipStreamSynchronize(st));
    }
    return FTK_OK;
}

ftk_status ftk_kmeans_fit(ftk_dtype dtype, const void *X, int64_t N, int32_t D, int32_t K,
                          int32_t iters, uint64_t seed, const void *C_init, void *C_out,
                          int32_t *labels_out, int32_t *counts_out, double *inertia_per_iter,
                          ftk_ft_mode ft, ftk_ft_stats *stats, void *workspace,
                          size_t workspace_bytes, void *hip_stream)
{
    return fit_impl(dtype, X, N, D, K, iters, seed, C_init, C_out, labels_out, counts_out, inertia_per_iter, ft,
                    stats, workspace, workspace_bytes, hip_stream, false);
}

ftk_status ftk_kmeans_fit_fast(ftk_dtype dtype, const void *X, int64_t N, int32_t D, int32_t K,
                               int32_t iters, uint64_t seed, const void *C_init, void *C_out,
                               int32_t *labels_out, int32_t *counts_out, double *inertia_per_iter,
                               ftk_ft_mode ft, ftk_ft_stats *stats, void *workspace, size_t workspace_bytes,
                               void *hip_stream)
{
    return fit_impl(dtype, X, N, D, K, iters, seed, C_init, C_out, labels_out, counts_out, inertia_per_iter, ft,
                    stats, workspace, workspace_bytes, hip_stream, true);
}

}  // extern "C"
