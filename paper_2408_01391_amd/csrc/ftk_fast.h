// Shared by the two split-bf16 assignment kernels (rows of up to 32 features: three pieces per
// operand; wider rows: two pieces): kernel arguments and the plan / launch hooks of the wide one.
#pragma once

#include "ftk_internal.h"
#include "ftk_mma.h"

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
    // fault tolerance / injection (as in the fp32 small-D kernel)
    ftk_ft_stats *stats;
    const float *chk_v1;  // [tiles_total*2][D8] plain checksum rows per (tile, lane group)
    const float *chk_v2;  // [tiles_total*2][D8] weighted (1..15) checksum rows
    const float *chk_s;   // [tiles_total*2][2]  matching sums of the half norms
    const ftk_fault *faults;
    int n_faults;
    int ft_mode;
    double ft_coef;       // detection threshold = ft_coef * (||x|| max||c|| + max||c||^2/2)
    float widen;          // 1 in strict mode, else 0
};

// rows of 33 .. 128 features (ftk_assign_fast_wide.hip)
size_t fast_wide_split_bytes(int D, int K);
void plan_fast_wide(int64_t N, int D, int K, ftk_ft_mode ft, AssignPlan &p);
ftk_status launch_assign_fast_wide(const AssignCall &c, const AssignPlan &p, const Workspace &w, hipStream_t st);

}  // namespace ftk
