// Matrix-instruction traits for gfx950 and small device helpers (internal).
//
// Orientation used throughout: the A operand holds CENTROIDS (output rows, spread over the
// accumulator registers of a lane), the B operand holds POINTS (output columns, one per
// lane).  A lane therefore owns one point and sees that point's scores against several
// centroids in its own registers, so the running arg-max of the fused epilogue
// (paper Sections 3.1.3-3.1.5) and the per-point checksums (Section 4) need no cross-lane
// traffic until the very end.
//
// Lane layouts (established with a probe on hardware; any mistake breaks the parity tests):
//   v_mfma_f32_32x32x2_f32 : lane l supplies A[l%32][l/32] and B[l/32][l%32];
//                            register r of lane l holds D[8*(r/4) + 4*(l/32) + r%4][l%32].
//   v_mfma_f64_16x16x4_f64 : lane l supplies A[l%16][l/16] and B[l/16][l%16];
//                            register r of lane l holds D[4*r + l/16][l%16].
// The contraction index may be permuted freely as long as both operands use the same
// permutation: lane group g = l/TN takes features 8q + E*g .. 8q + E*g + E-1 of "quad" q
// (8 consecutive features), which makes every operand fetch one aligned 16-byte access.
#pragma once

#include <hip/hip_runtime.h>

namespace ftk {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef double doublex4 __attribute__((ext_vector_type(4)));
typedef double doublex2 __attribute__((ext_vector_type(2)));

template <typename T>
struct Mma;

template <>
struct Mma<float> {
    static constexpr int TM = 32;  // centroids per tile
    static constexpr int TN = 32;  // points per tile
    static constexpr int G = 2;    // lane groups sharing a point
    static constexpr int R = 16;   // accumulator registers per lane per tile
    static constexpr int E = 4;    // elements per 16-byte fragment
    using acc_t = floatx16;
    using frag_t = floatx4;
    static constexpr double kEps = 5.9604644775390625e-08;  // 2^-24
    static __device__ __forceinline__ int row(int r, int g) { return 8 * (r >> 2) + 4 * g + (r & 3); }
    static __device__ __forceinline__ acc_t mma(float a, float b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ float med3(float a, float b, float c)
    {
        return __builtin_amdgcn_fmed3f(a, b, c);
    }
    static __device__ __forceinline__ float neg_inf() { return -__builtin_huge_valf(); }
    static __device__ __forceinline__ float huge() { return __builtin_huge_valf(); }
};

template <>
struct Mma<double> {
    static constexpr int TM = 16;
    static constexpr int TN = 16;
    static constexpr int G = 4;
    static constexpr int R = 4;
    static constexpr int E = 2;
    using acc_t = doublex4;
    using frag_t = doublex2;
    static constexpr double kEps = 1.1102230246251565e-16;  // 2^-53
    static __device__ __forceinline__ int row(int r, int g) { return 4 * r + g; }
    static __device__ __forceinline__ acc_t mma(double a, double b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ double med3(double a, double b, double c)
    {
        // median of three; callers pass a >= b
        return fmax(b, fmin(a, c));
    }
    static __device__ __forceinline__ double neg_inf() { return -__builtin_huge_val(); }
    static __device__ __forceinline__ double huge() { return __builtin_huge_val(); }
};

// E consecutive elements of a row starting at feature d0, zero beyond D.
template <typename T, bool ALIGNED>
__device__ __forceinline__ typename Mma<T>::frag_t load_frag(const T *row, int d0, int D)
{
    using F = typename Mma<T>::frag_t;
    F f;
    if constexpr (ALIGNED) {
        if (d0 < D) {
            f = *reinterpret_cast<const F *>(row + d0);
        } else {
#pragma unroll
            for (int e = 0; e < Mma<T>::E; ++e) f[e] = T(0);
        }
    } else {
#pragma unroll
        for (int e = 0; e < Mma<T>::E; ++e) f[e] = (d0 + e < D) ? row[d0 + e] : T(0);
    }
    return f;
}

// Branch-free variant for the hot loops: the access is clamped into the row, so elements at or
// beyond D come back as copies of valid elements of the same row (finite whenever the row is).
// A load inside a branch would force the compiler to wait for every outstanding load at the next
// use; callers either multiply the surplus elements by zero or clear them with frag_keep().
template <typename T, bool ALIGNED>
__device__ __forceinline__ typename Mma<T>::frag_t load_frag_clamped(const T *row, int d0, int D)
{
    using F = typename Mma<T>::frag_t;
    constexpr int E = Mma<T>::E;
    if constexpr (ALIGNED) {
        return *reinterpret_cast<const F *>(row + min(d0, D - E));
    } else {
        F f;
#pragma unroll
        for (int e = 0; e < E; ++e) f[e] = row[min(d0 + e, D - 1)];
        return f;
    }
}

// Keeps element e of a fragment fetched at feature d0 if `keep` and d0 + e < D, else zero.
template <typename T>
__device__ __forceinline__ typename Mma<T>::frag_t frag_keep(typename Mma<T>::frag_t f, int d0, int D, bool keep)
{
#pragma unroll
    for (int e = 0; e < Mma<T>::E; ++e) f[e] = (keep && d0 + e < D) ? f[e] : T(0);
    return f;
}

// Squared distance in the direct-difference form of the basic kernel (Section 3.1.1),
// accumulated in double.  Used to settle points whose best scores are closer than the
// rounding-error bound of the expanded form.
// Features are added in index order into one accumulator (so two candidates evaluated here
// always compare consistently, and identical centroids tie exactly); the loads are issued
// several fragments ahead, since their latency - not the arithmetic - is what a lane waits for.
template <typename T, bool ALIGNED>
__device__ __forceinline__ double exact_sqdist(const T *x, const T *c, int D)
{
    constexpr int E = Mma<T>::E;
    double s = 0.0;
#pragma unroll 4
    for (int d0 = 0; d0 < D; d0 += E) {
        const typename Mma<T>::frag_t xf = load_frag<T, ALIGNED>(x, d0, D);
        const typename Mma<T>::frag_t cf = load_frag<T, ALIGNED>(c, d0, D);
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const double diff = (double)xf[e] - (double)cf[e];
            s = fma(diff, diff, s);
        }
    }
    return s;
}

// Running best-three scores and best-two indices of one point.
template <typename T>
struct Top3 {
    T m1, m2, m3;
    int i1, i2;
};

// Insert score s (centroid j).  Written on by-value locals so that every choice is a select
// (v_cndmask) rather than a branch.
template <typename T>
__device__ __forceinline__ Top3<T> top3_insert(Top3<T> b, T s, int j)
{
    const T m1 = b.m1, m2 = b.m2, m3 = b.m3;
    const int i1 = b.i1, i2 = b.i2;
    const bool c1 = s > m1;
    const bool c2 = s > m2;
    const int i2a = c2 ? j : i2;
    Top3<T> o;
    o.i2 = c1 ? i1 : i2a;
    o.i1 = c1 ? j : i1;
    o.m3 = Mma<T>::med3(m2, m3, s);
    o.m2 = Mma<T>::med3(m1, m2, s);
    o.m1 = c1 ? s : m1;
    return o;
}

// Append this lane's point to the refine work-list if `need`; one atomic per wave.
__device__ __forceinline__ void worklist_push(bool need, int32_t point, int32_t *wl, int32_t *wl_count)
{
    const unsigned long long m = __ballot(need);
    if (m == 0ull) return;
    const int lane = (int)(threadIdx.x & 63);
    const int leader = __ffsll((long long)m) - 1;
    int base = 0;
    if (lane == leader) base = atomicAdd(wl_count, (int)__popcll(m));
    base = __shfl(base, leader, 64);
    if (need) wl[base + (int)__popcll(m & ((1ull << lane) - 1ull))] = point;
}

__device__ __forceinline__ float shfl_xor_t(float v, int m) { return __shfl_xor(v, m, 64); }
__device__ __forceinline__ double shfl_xor_t(double v, int m) { return __shfl_xor(v, m, 64); }
__device__ __forceinline__ int shfl_xor_t(int v, int m) { return __shfl_xor(v, m, 64); }

}  // namespace ftk
