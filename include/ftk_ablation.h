/*
 * ftk_ablation.h -- the earlier steps of the paper's stepwise optimisation (Section 3.1, the
 * stepwise figure of Section 5.1), kept as separately built measurement kernels so that the
 * fused matrix-core kernel of ftkmeans.h can be placed against what it replaces:
 *
 *   naive         the basic kernel of Section 3.1.1: one thread per point walks all K
 *                 centroids and all D features (direct-difference form) and keeps the minimum;
 *   gemm_unfused  variant V1 of Section 3.1.2: centroid norms, the product X C^T from the
 *                 vendor GEMM (rocBLAS) written to memory in full, and a separate kernel that
 *                 reads it back to take the per-point arg-min;
 *   fused_alu     variants V2 and V3 of Sections 3.1.3 and 3.1.4: a register-tiled GEMM on the
 *                 plain (non-matrix-core) ALUs whose epilogue takes the minimum at thread and
 *                 threadblock level, so the product is never stored.  V2 leaves one candidate
 *                 per point and block of 128 centroids and reduces them in a second kernel;
 *                 V3 merges the candidates of all centroid blocks with one device-wide atomic
 *                 minimum per point on a packed (distance, index) word.
 *
 * These are not part of the product path (libftkmeans.so neither links nor calls them).
 * Conventions as in ftkmeans.h: device pointers owned by the caller, row-major X [N x D] and
 * C [K x D], squared distances, lowest index on exact ties, work only enqueued on `hip_stream`,
 * errors by return code (0 = ok, 1 = invalid argument, 3 = workspace too small, 4 = device or
 * library failure) with ftk_abl_last_error() giving the text.
 *
 * The unfused variant decides in the working precision from the expanded form, so on data whose
 * norms are large against the nearest distance its labels can differ from the exact arg-min
 * where two candidates are closer than the rounding error of that form; the naive variant
 * decides from the direct form and differs only on near-exact ties.
 */
#ifndef FTK_ABLATION_H
#define FTK_ABLATION_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* dtype: 0 = fp32, 1 = fp64.  labels [N] int32 out; mindist [N] (working precision) out,
 * may be NULL. */
int ftk_abl_naive_assign(int dtype, const void *X, const void *C, int64_t N, int32_t D, int32_t K,
                         int32_t *labels, void *mindist, void *hip_stream);

/* Bytes of device scratch ftk_abl_gemm_assign needs: the [N x K] product plus the K norms. */
size_t ftk_abl_gemm_workspace_bytes(int dtype, int64_t N, int32_t K);

/* The first call creates a rocBLAS handle for the calling process (this allocates and may take
 * seconds); later calls reuse it.  One handle is shared: do not call from several threads at
 * once.  The GEMM interface takes 32-bit extents, so N must be below 2^31. */
int ftk_abl_gemm_assign(int dtype, const void *X, const void *C, int64_t N, int32_t D, int32_t K,
                        int32_t *labels, void *mindist, void *workspace, size_t workspace_bytes,
                        void *hip_stream);

/* Bytes of device scratch ftk_abl_fused_alu_assign needs: the K norms plus, for variant 2, the
 * [N][ceil(K/128)] candidate values and indices, or, for variant 3, one 64-bit word per point. */
size_t ftk_abl_fused_alu_workspace_bytes(int dtype, int64_t N, int32_t K, int32_t variant);

/* variant: 2 (both dtypes) or 3 (fp32 only: its atomic key packs a 32-bit distance with the
 * index; fp64 with variant 3 returns 1).  Decides from the expanded form in the working
 * precision, like the unfused variant. */
int ftk_abl_fused_alu_assign(int dtype, const void *X, const void *C, int64_t N, int32_t D, int32_t K,
                             int32_t *labels, void *mindist, int32_t variant, void *workspace,
                             size_t workspace_bytes, void *hip_stream);

/* One bf16 matrix instruction (v_mfma_f32_32x32x16_bf16) per problem on plain matrices, all device
 * pointers: D = A B + C with A [tiles][32][16] and B [tiles][16][32] as bf16 bit patterns, C and D
 * [tiles][32][32] fp32, row-major.  A probe for tests: the error bound of the reduced-precision
 * assignment (the counterpart of the TF32 path of Section 3.1.5) is built on how this instruction
 * rounds, which only measurement tells. */
int ftk_abl_mfma_bf16(const uint16_t *A, const uint16_t *B, const float *C, float *D, int32_t tiles,
                      void *hip_stream);

/* The same for the instructions of the main path: v_mfma_f32_32x32x2_f32 (A [tiles][32][2],
 * B [tiles][2][32], C and D [tiles][32][32]) and v_mfma_f64_16x16x4_f64 (A [tiles][16][4],
 * B [tiles][4][16], C and D [tiles][16][16]).  The rounding band of the assignment (twice (D+4) u
 * of the magnitude) assumes a chain of fused multiply-adds over the contraction index in order. */
int ftk_abl_mfma_f32(const float *A, const float *B, const float *C, float *D, int32_t tiles, void *hip_stream);
int ftk_abl_mfma_f64(const double *A, const double *B, const double *C, double *D, int32_t tiles,
                     void *hip_stream);

const char *ftk_abl_last_error(void);

#ifdef __cplusplus
}
#endif
#endif
