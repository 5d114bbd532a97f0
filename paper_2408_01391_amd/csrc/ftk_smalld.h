// Pieces shared by the small-D assignment kernels (fp32 matrix path and the split-bf16 fast path):
// tile geometry, the one-instruction maxima, the exact re-evaluation of a group of rows, and the
// per-lane record of the best tile.
#pragma once

#include "ftk_internal.h"
#include "ftk_mma.h"

namespace ftk {

__device__ __forceinline__ float max3f(float a, float b, float c) { return __builtin_fmaxf(__builtin_fmaxf(a, b), c); }
// max(a, b) of values below FLT_MAX as the median of (a, b, FLT_MAX): one instruction, where
// fmaxf() spends two more on canonicalising its operands (with +inf as the third operand the
// compiler turns it back into fmaxf).  A NaN operand gives NaN, which later sends the point to
// the exact recomputation.
__device__ __forceinline__ float max2f(float a, float b) { return __builtin_amdgcn_fmed3f(a, b, 3.402823466e38f); }

// Tile geometry: which centroid sits in register r of lane group g of tile T.
template <bool FT>
struct TileGeom {
    static constexpr int CPT = FT ? 30 : 32;  // centroids per tile
    static constexpr int RG = FT ? 15 : 16;   // score registers per lane group
    static __device__ __forceinline__ int centroid(int T, int g, int r)
    {
        return FT ? 30 * T + 15 * g + r : 32 * T + Mma<float>::row(r, g);
    }
};

// Exact (direct-difference, fp32) distances of one point to 8 centroids: registers r0..r0+7 of
// lane group gw in tile T, whose LDS / global rows start at `base` (`stride` floats per row).
// xlo / xhi hold features 8q..8q+3 and 8q+4..8q+7 of the point, so terms are always added in
// feature order and identical centroids give bit-identical distances whichever lane evaluates
// them.  Keeps the running (distance, index) minimum, lowest index on equal distance.
// LDSROWS: rows are addressed by their position in the staged tile and are zero-padded to
// 8*NQ features; otherwise rows are addressed by centroid index in global C.
template <int NQ, bool FT, bool LDSROWS>
__device__ __forceinline__ void eval_rows(const floatx4 (&xlo)[NQ], const floatx4 (&xhi)[NQ],
                                          const float *base, int stride, int T, int K, int D,
                                          int gw, int r0, float &dbest, int &jbest)
{
    // rows in register order, the running minimum updated as they come; with many features the
    // loop is unrolled only twice (all eight rows in flight would need more registers than exist)
    constexpr int UNROLL = NQ == 1 ? 4 : (NQ == 2 ? 8 : 2);
#pragma unroll UNROLL
    for (int i = 0; i < 8; ++i) {
        // register r = r0 + i of group gw holds tile row 8*(r/4) + 4*gw + r%4; r0 is 0 or 8
        const int row = 8 * (i >> 2) + (i & 3) + 2 * r0 + 4 * gw;
        const bool real = FT ? (r0 + i < 15) : true;
        const int j = FT ? 30 * T + 15 * gw + r0 + i : 32 * T + row;
        const int jj = (real && j < K) ? j : 0x7fffffff;
        const float *c = LDSROWS ? base + row * stride : base + (size_t)(j < K ? j : 0) * stride;
        float d = 0.f;
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            floatx4 cl = {0.f, 0.f, 0.f, 0.f}, ch = {0.f, 0.f, 0.f, 0.f};
            if (LDSROWS || 8 * q < D) cl = *reinterpret_cast<const floatx4 *>(c + 8 * q);
            if (LDSROWS || 8 * q + 4 < D) ch = *reinterpret_cast<const floatx4 *>(c + 8 * q + 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float t = xlo[q][e] - cl[e];
                d = fmaf(t, t, d);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float t = xhi[q][e] - ch[e];
                d = fmaf(t, t, d);
            }
        }
        const float db = dbest;
        const int jb = jbest;
        const bool better = (jj != 0x7fffffff) & ((d < db) | ((d == db) & (jj < jb)));
        dbest = better ? d : db;
        jbest = better ? jj : jb;
    }
}

constexpr int SMALLD_MAX_FAULTS = 4;  // injected faults honoured per point block

// Sum of the 15 scores of one lane group, added pairwise: partial sums stay small, which roughly
// halves the rounding noise of a running sum (and the four sub-sums are independent chains).
__device__ __forceinline__ float sum15(const floatx16 &a)
{
    const float p0 = (a[0] + a[1]) + (a[2] + a[3]);
    const float p1 = (a[4] + a[5]) + (a[6] + a[7]);
    const float p2 = (a[8] + a[9]) + (a[10] + a[11]);
    const float p3 = (a[12] + a[13]) + a[14];
    return (p0 + p1) + (p2 + p3);
}

// Work-list entries of a workgroup are collected in LDS: one device-wide atomic per wave of
// entries when they are handed over, instead of one per wave and point tile (tens of thousands of
// atomics on one word keep a dispatch open long after its last wave).  A wave that finds the
// buffer full appends to the global list directly.
constexpr int SMALLD_LIST_CAP = 512;
__device__ __forceinline__ void block_list_push(bool need, int32_t point, int32_t *sh_list, int *sh_count,
                                                int32_t *wl, int32_t *wl_count)
{
    const unsigned long long m = __ballot(need);
    if (m == 0ull) return;
    const int lane = (int)(threadIdx.x & 63);
    const int leader = __ffsll((long long)m) - 1;
    const int n = (int)__popcll(m);
    int base = 0;
    if (lane == leader) base = atomicAdd(sh_count, n);
    base = __shfl(base, leader, 64);
    if (base + n <= SMALLD_LIST_CAP) {
        if (need) sh_list[base + (int)__popcll(m & ((1ull << lane) - 1ull))] = point;
    } else {
        worklist_push(need, point, wl, wl_count);
    }
}

// Best tile maximum, the tile it came from, and the runner-up tile maximum of one lane.
struct TileBest {
    float m1, m2;
    int t1;
};

}  // namespace ftk
