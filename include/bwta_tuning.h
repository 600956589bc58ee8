/*
 * bwta_tuning.h -- benchmark and tuning hooks of libbwta.so.  Not part of the layer's contract
 * (bwta.h): nothing here changes a result, only which kernel instance computes it.  The settings
 * are process-wide atomics; a launch uses the values it reads when it is enqueued.
 */
#ifndef BWTA_TUNING_H
#define BWTA_TUNING_H

#ifdef __cplusplus
extern "C" {
#endif

/* Which family AUTO resolves to for a shape: BWTA_PATH_POPC, BWTA_PATH_MFMA or BWTA_PATH_FP4. */
int bwta_auto_path(int M, int N, int K);
/* Which contraction kernel a product of this shape is dispatched to under the current path setting
 * (a pure host function: nothing is launched).  operand = 0: canonical planes with a workspace
 * (bwta_gemm); BWTA_PREPARED_PLANES or BWTA_PREPARED_FP4: bwta_gemm_prepared with that format.
 * Prepared planes never resolve to BWTA_KERNEL_GEMM_FP4: that kernel needs scratch for its
 * fragments and bwta_gemm_prepared has none.  0 for a non-positive dimension or an unknown operand. */
enum {
    BWTA_KERNEL_GEMV_POPC = 1,    /* decode, wave64 popcount            */
    BWTA_KERNEL_GEMV_FP4 = 2,     /* decode, FP4 matrix cores           */
    BWTA_KERNEL_GEMM_FP4 = 3,     /* tiled, FP4 matrix cores            */
    BWTA_KERNEL_GEMM_MFMA_I8 = 4, /* tiled, int8 matrix cores (planes)  */
    BWTA_KERNEL_GEMM_POPC = 5     /* tiled, wave64 popcount (planes)    */
};
int bwta_planned_kernel(int operand, int M, int N, int K);
/* How many kernels bwta_linear launches for a shape under the current settings, given a dense
 * (lda = K), 16-byte-aligned fp16 input: 1 where ternarisation, product and epilogue run as one
 * kernel (short K), else 2.  Informational (benchmarks label their timings with it); 0 for a
 * non-positive dimension. */
int bwta_linear_launches(int M, int N, int K);
/* Tuning hook for benchmark sweeps: force the FP4 kernel's per-wavefront tile (22, 21, 12, 11, 13
 * = blocks of 32 rows x 32 columns per wavefront; 23 = 22 at three wavefronts per SIMD; 222 = 22
 * with K split over two groups of wavefronts; 243, 223, 323 = the kernel that stages both operands
 * through LDS with direct loads, as 128 x 256 tiles of 8 wavefronts, 128 x 128 tiles of 4, or
 * 128 x 256 tiles of 4 wavefronts of 64 tokens x 128 channels), the popcount decode kernel's row split (1000 + 16 *
 * lanes per row (8, 16, 32) + chunks per lane; ignored where the registers cannot hold it) or the
 * matrix-core decode kernel's work split (2000 + 1024 * ring depth (2..4) + 64 * chunks per
 * wavefront (1..4) + tiles per workgroup (rounded up to a multiple of the ring depth, fewer if LDS
 * does not hold their partials)), or where bwta_linear runs as a single launch (900 never, 901
 * wherever the one-launch kernel can run, 900 + R the same with R channel splits per token
 * strip); 0 restores the built-in choices.  Results do not depend on it. */
int bwta_set_tile(int tile);
#ifdef __cplusplus
}
#endif
#endif /* BWTA_TUNING_H */
