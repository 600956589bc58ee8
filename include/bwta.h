/*
 * bwta.h -- C ABI of the BWTA (Binary Weights & Ternary Activations) linear-layer
 * hot path for AMD MI355X (gfx950).
 *
 * The layer is the paper's BWTA linear equation ("Basic Layers for Linear and
 * MatMul"):   linear(A) = s_W * s_A * ( sign(W) (x) ternary(A^T, s_A) ),
 * evaluated the way its kernel section describes: binary weights are packed to
 * one bit each ahead of time, activations are ternarised and packed to two bit
 * planes at run time, the product is an exact integer contraction with int32
 * accumulation, and results are cast back to fp16 before they leave the kernel.
 *
 * Conventions shared by every call
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *     allocates nothing, frees nothing, keeps no pointer after the call returns
 *     and never synchronises: work is enqueued on `stream` (a hipStream_t passed
 *     as void*; NULL is the null stream) and the call returns at once.
 *   - Matrices are row-major.  Activations are [M, K] (M tokens), weights are
 *     [N, K] (N output channels), results are [M, N]; the paper writes the same
 *     numbers as W (x) A^T, i.e. transposed.
 *   - Packed planes: element k of a row sits in 32-bit word k/32 at bit k%32
 *     (least significant bit first).  Rows hold bwta_plane_row_words(K) words,
 *     i.e. they are padded with ZERO bits to a multiple of 128 bits, and plane
 *     base pointers must be 16-byte aligned.  Polarity follows the paper's
 *     bitpack: a negative value is bit 1, a positive value bit 0.  A ternary
 *     operand uses two planes: `mask` (value != 0) and `sign` (value < 0, always
 *     a subset of mask); the paper's A- plane is `sign`, its A+ plane is
 *     mask ^ sign.
 *   - Scales are fp16.  scale_mode says how a scale pointer is read:
 *     BWTA_SCALE_NONE (pointer ignored, scale 1), BWTA_SCALE_SCALAR (one value),
 *     BWTA_SCALE_VECTOR (one per token for s_a, one per output channel for s_w).
 *   - Return value: BWTA_OK, or a negative BWTA_ERR_* code.  Argument errors are
 *     detected on the host before anything is enqueued; BWTA_ERR_HIP means a
 *     launch was rejected by the runtime (see bwta_last_hip_error()).
 */
#ifndef BWTA_H
#define BWTA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef void *bwta_stream_t; /* a hipStream_t */

enum {
    BWTA_OK = 0,
    BWTA_ERR_NULL = -1,        /* a required pointer is NULL                               */
    BWTA_ERR_SHAPE = -2,       /* M, N or K < 0, K == 0 with M,N > 0, or a leading dim < row */
    BWTA_ERR_ALIGN = -3,       /* a plane / output pointer or leading dimension is misaligned */
    BWTA_ERR_UNSUPPORTED = -4, /* unknown dtype, scale mode or path                        */
    BWTA_ERR_WORKSPACE = -5,   /* workspace NULL or smaller than bwta_workspace_bytes()    */
    BWTA_ERR_HIP = -6,         /* the HIP runtime reported an error at launch              */
    BWTA_ERR_TOO_LARGE = -7    /* bwta_linear_static: the shape needs more than the static scratch */
};

enum { BWTA_DTYPE_FP16 = 0, BWTA_DTYPE_INT8 = 1 };
enum { BWTA_SCALE_NONE = 0, BWTA_SCALE_SCALAR = 1, BWTA_SCALE_VECTOR = 2 };
/* Which contraction kernel bwta_gemm / bwta_linear use.  AUTO picks per shape regime from
 * measurements on MI355X; the others force the wave64 popcount kernels, the int8 matrix-core
 * (MFMA) kernel that widens bit planes to int8, or the FP4 matrix-core kernel (+-1 and 0 are
 * exact in E2M1).  All of them produce identical bits. */
enum { BWTA_PATH_AUTO = 0, BWTA_PATH_POPC = 1, BWTA_PATH_MFMA = 2, BWTA_PATH_FP4 = 3 };

/* Words per packed row: 4 * ceil(K / 128).  Returns 0 for K <= 0. */
int64_t bwta_plane_row_words(int K);

/* Bytes of caller-provided scratch that bwta_linear (and bwta_gemm) need for this shape;
 * a pure function of (M, N, K), 256-byte granular, 0 only if M, N or K is 0. */
size_t bwta_workspace_bytes(int M, int N, int K);

/*
 * Ternarise and bit-pack activations (the paper's "Ternary Function" equation, packed as in
 * "Instruction-level Parallel Bitpack" / ternary bitpack).
 *   A        a_dtype FP16: fp16 [M, lda]; element -> +1 if a >= 0.5*s, -1 if a < -0.5*s,
 *            else 0 (so a == +0.5*s gives +1 and a == -0.5*s gives 0, as printed).  The
 *            comparison is exact (no division).  NaN gives 0, +-Inf gives +-1.  A scale that is
 *            not finite and > 0 ternarises its row to 0.
 *            a_dtype INT8: int8 [M, lda] already ternary; >0 -> +1, <0 -> -1 (scale unused).
 *   lda      leading dimension in elements, >= K.
 *   s_a      fp16 scale(s) per scale_mode (per token for VECTOR); may be NULL with NONE.
 *   mask, sign   out, u32 [M, row_words] each, pad bits written as 0.
 *   nnz      out, optional (NULL to skip): int32 [M], nonzeros per token.
 */
int bwta_quantize_pack_act(const void *A, int a_dtype, int64_t lda, const void *s_a,
                           int scale_mode, int M, int K, uint32_t *mask, uint32_t *sign,
                           int32_t *nnz, bwta_stream_t stream);

/*
 * Sign-pack binary weights (the paper's sign equation in "Binary Functions"; done once, before
 * inference).  W is fp16 [N, ldw] (bit = 0 if w >= 0, so -0.0 -> bit 0; otherwise, NaN
 * included, bit 1) or int8 [N, ldw] (bit = w < 0).  wsign: out, u32 [N, row_words].
 * Mean-centring and the weight scale are the caller's business: pass W - mean(W) and keep s_W.
 */
int bwta_pack_weights(const void *W, int w_dtype, int64_t ldw, int N, int K, uint32_t *wsign,
                      bwta_stream_t stream);

/*
 * BWTA matrix product with fused scale epilogue (Case 1 of the paper's "Comprehensive
 * Computational Implementations", the xor-based BWTA MatMul):
 *   acc[m, n] = sum_k t[m,k] * w[n,k] = popc(mask_m) - 2 * popc(mask_m & (sign_m ^ wsign_n))
 *   out[m, n] = fp16( s_w[n] * s_a[m] * acc[m, n] )   exact product, one rounding (nearest even)
 *   mask, sign  u32 [M, row_words]; sign bits under a zero mask bit are ignored.  mask == NULL
 *               means binary (+-1) activations, every element non-zero: the W1A1 "Binary Linear"
 *               special case acc = K - 2 * popc(sign_m ^ wsign_n); pack such activations with
 *               bwta_pack_weights (the sign packer).  No mask plane is read; kernels that need
 *               one get it built in the workspace.
 *   wsign       u32 [N, row_words].
 *   s_a, s_w    fp16 scales read per a_scale_mode / w_scale_mode (one per token / per channel with
 *               VECTOR, one value with SCALAR, ignored with NONE).
 *   acc         optional out, int32 [M, N] dense (leading dimension N).
 *   out         optional out, fp16 [M, ldo], ldo >= N.  At least one of acc / out.
 *   workspace   scratch of at least bwta_workspace_bytes(M, N, K) bytes, 256-byte aligned;
 *               contents undefined afterwards.  Calls that share a workspace must not overlap.
 */
int bwta_gemm(const uint32_t *mask, const uint32_t *sign, const uint32_t *wsign, int M, int N,
              int K, const void *s_a, int a_scale_mode, const void *s_w, int w_scale_mode,
              int32_t *acc, void *out, int64_t ldo, void *workspace, size_t workspace_bytes,
              bwta_stream_t stream);

/*
 * The whole layer on fp16 activations: ternarise + pack + product + scale epilogue
 * (the BWTA linear equation end to end).  A fp16 [M, lda]; wsign from bwta_pack_weights;
 * out fp16 [M, ldo].  s_a is used both as the ternarisation scale and in the epilogue.
 * Runs as two kernels (ternarise into the workspace, then the product) or, for short K
 * (at most 1024) with 16-byte-aligned rows and at least two tokens, as one kernel that never
 * touches the workspace;
 * the result is the same bit for bit (see bwta_linear_launches).  The workspace is required
 * either way.
 */
int bwta_linear(const void *A, int64_t lda, const void *s_a, int a_scale_mode,
                const uint32_t *wsign, const void *s_w, int w_scale_mode, int M, int N, int K,
                void *out, int64_t ldo, void *workspace, size_t workspace_bytes,
                bwta_stream_t stream);

/*
 * bwta_linear for callers that cannot allocate or pass a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the same
 * bits as bwta_linear, except that the scratch is an array inside the library's own device image
 * (BWTA_STATIC_SCRATCH_BYTES on every GPU the library is used on, held until the process ends)
 * instead of a caller buffer.  The call allocates nothing and frees nothing.
 *   - A shape with bwta_workspace_bytes(M, N, K) > BWTA_STATIC_SCRATCH_BYTES is refused with
 *     BWTA_ERR_TOO_LARGE before anything is enqueued (32 MiB covers e.g. 2048 tokens at K = 11008
 *     and 4096 tokens at K = 3072).
 *   - All calls on one GPU share that GPU's array: calls that may overlap on the same GPU (two
 *     streams, two threads) race; serialise them or use bwta_linear with separate workspaces.
 *     Nothing in the array has to be cleared between calls.
 *   - The array's address is looked up once per device (hipGetSymbolAddress, with that device
 *     current) on the first call there; bwta_static_scratch_init() does the look-up for the current
 *     device ahead of time, e.g. before a graph capture starts.  Both return BWTA_ERR_HIP if the
 *     look-up fails.
 */
#define BWTA_STATIC_SCRATCH_BYTES (32u << 20)
size_t bwta_static_scratch_bytes(void);
int bwta_static_scratch_init(void);
int bwta_linear_static(const void *A, int64_t lda, const void *s_a, int a_scale_mode,
                       const uint32_t *wsign, const void *s_w, int w_scale_mode, int M, int N, int K,
                       void *out, int64_t ldo, bwta_stream_t stream);

/*
 * The two halves of bwta_linear as separate calls, so that one ternarisation can feed several
 * weight matrices (Q/K/V, gate/up): bwta_prepare_act ternarises fp16 activations (same rule and
 * arguments as bwta_quantize_pack_act with FP16 input) into `prepared`, a device buffer of
 * bwta_prepared_bytes(M, K) bytes, 256-byte aligned, and writes to *prepared_format (a HOST int,
 * required) which of two layouts it chose there: BWTA_PREPARED_PLANES (the two canonical bit
 * planes, for the decode-sized kernels) or BWTA_PREPARED_FP4 (E2M1 fragments in matrix-core operand
 * order, for the tiled kernel).  The choice depends on M, K and the path setting at the time of the
 * call (bwta_prepared_format tells it in advance).  bwta_gemm_prepared takes that format id back
 * and computes out = fp16(s_w * s_a * (sign(W) (x) ternary(A))) exactly like bwta_gemm, with a
 * kernel that reads that layout: the format id, not the path setting at the time of the second
 * call, says how `prepared` is read, so changing the path in between is harmless.  An id that is
 * neither of the two gives BWTA_ERR_UNSUPPORTED; passing the other layout's id reads the (other,
 * possibly unwritten) region of the caller's own buffer, never memory outside it.  With planes and
 * a shape the decode kernels do not cover, the product runs on the int8 matrix-core or popcount
 * kernels (same bits), since no scratch comes with this call.  `prepared` is only read by it.
 */
enum { BWTA_PREPARED_PLANES = 1, BWTA_PREPARED_FP4 = 2 };
size_t bwta_prepared_bytes(int M, int K);
int bwta_prepared_format(int M, int K);
int bwta_prepare_act(const void *A, int64_t lda, const void *s_a, int a_scale_mode, int M, int K,
                     void *prepared, size_t prepared_bytes, int *prepared_format, bwta_stream_t stream);
int bwta_gemm_prepared(const void *prepared, size_t prepared_bytes, int prepared_format,
                       const uint32_t *wsign, int M, int N, int K, const void *s_a, int a_scale_mode,
                       const void *s_w, int w_scale_mode, int32_t *acc, void *out, int64_t ldo,
                       bwta_stream_t stream);

/*
 * Several BWTA products of ONE shape in one call (a decode step's independent matrices, expert
 * groups, or a bandwidth measurement over many weight matrices).  `problems` is a HOST array of
 * `count` records of DEVICE pointers with the meaning they have in bwta_gemm; scale modes, ldo
 * and the workspace rule are shared (workspace: count * bwta_workspace_bytes(M, N, K) bytes,
 * 256-byte aligned).  For M <= 128 (decode and small batches) all problems run in one kernel
 * launch per 64 problems; otherwise the call is equivalent to `count` bwta_gemm calls.
 */
typedef struct bwta_gemm_problem {
    const uint32_t *mask, *sign, *wsign;
    const void *s_a, *s_w;
    int32_t *acc;
    void *out;
} bwta_gemm_problem;
int bwta_gemm_grouped(const bwta_gemm_problem *problems, int count, int M, int N, int K,
                      int a_scale_mode, int w_scale_mode, int64_t ldo, void *workspace,
                      size_t workspace_bytes, bwta_stream_t stream);

/*
 * Boolean activations (the paper's bool function, used for attention probabilities and other
 * non-negative activations): bit k of word k / 32 of row m = 1 iff A[m, k] >= 0.5 * s (exact
 * compare, no division).  A is fp16 [M, lda]; scale rules as in bwta_quantize_pack_act (an
 * invalid scale clears the row; NaN -> 0; +Inf -> 1).  One plane [M, bwta_plane_row_words(K)],
 * pad bits zero; it is the `mask` of an operand with no sign plane.
 */
int bwta_quantize_pack_bool(const void *A, int64_t lda, const void *s_a, int scale_mode, int M, int K,
                            uint32_t *mask, bwta_stream_t stream);

/*
 * The attention MatMuls of the paper ("Basic Layers for Linear and MatMul": the BWTA_QK and
 * BWTA_Att rules; arithmetic Cases 3 and 2), batched over heads:
 *   acc[b, m, n] = sum_k a[b, m, k] * b[b, n, k]        a, b in {-1, 0, +1} given as bit planes
 *   out[b, m, n] = fp16( acc * fp32( alpha * (s_a * s_b) ) )   one rounding of the scale product
 *                                                              to fp32, one of the result to fp16
 * Both operands are K-major packed planes as produced by bwta_quantize_pack_act ([rows,
 * bwta_plane_row_words(K)] words, batches `strideA` / `strideB` words apart).  A NULL sign plane
 * means the operand is boolean (bwta_quantize_pack_bool): bool x ternary is the BWTA_Att rule
 * popc(Att & V+) - popc(Att & V-); two ternary operands give the BWTA_QK rule.  For Q K^T pass
 * Q as A [S, D] and K as B [S, D] with alpha = 1 / sqrt(D); for Att V pass Att as A [S, S] and V
 * TRANSPOSED ([D, S], packed along the sequence) as B.
 *   s_a, s_b   fp16 scales; VECTOR means one per row of every batch ([batch, M] / [batch, N]).
 *   acc        optional int32 [batch, M, N] (dense); out optional fp16, row stride ldo >= N,
 *              batches stride_out elements apart.  At least one of acc / out.
 * Runs on the FP4 matrix cores (+-1 and 0 are exact E2M1 values; fp32 accumulation of integers
 * below 2^24 is exact); bwta_set_path(BWTA_PATH_POPC) selects the wave64 popcount kernel
 * instead.  Both give identical bits.
 * Errors as bwta_gemm; nothing is enqueued on error.
 */
int bwta_matmul_tt(const uint32_t *maskA, const uint32_t *signA, int64_t strideA, const uint32_t *maskB,
                   const uint32_t *signB, int64_t strideB, int batch, int M, int N, int K, const void *s_a,
                   int a_scale_mode, const void *s_b, int b_scale_mode, float alpha, int32_t *acc, void *out,
                   int64_t ldo, int64_t stride_out, bwta_stream_t stream);

/*
 * The BWTA_Att rule (bool x ternary, arithmetic Case 2) with the ternary operand prepared once:
 *   acc[b, m, n] = sum_k A[b, m, k] * B[b, n, k]      A boolean: its plane from
 *                                                     bwta_quantize_pack_bool, [M, row_words] per
 *                                                     batch entry, entries strideA words apart
 *   out[b, m, n] = fp16( acc * fp32( alpha * (s_a * s_b) ) )   as bwta_matmul_tt
 * B is `preparedB`: what bwta_prepare_act wrote for the fp16 matrix [batch * N, K] that stacks the
 * batch entries' N rows (for Att V: V transposed, [heads * D, S]), with the format id it reported.  The boolean plane then plays the
 * part the packed weights play in bwta_gemm_prepared, which is several times cheaper per product
 * than expanding both operands from planes (bwta_matmul_tt).  Same bits as bwta_matmul_tt.
 * Needs N a multiple of 128 and preparedB_format == BWTA_PREPARED_FP4 (which bwta_prepare_act
 * chooses on the FP4 path, AUTO included, above 128 rows); BWTA_ERR_UNSUPPORTED otherwise.  out fp16 [batch][M][ldo], ldo >= N,
 * entries stride_out elements apart; s_a [batch, M] / s_b [batch, N] when VECTOR.
 */
int bwta_matmul_bool_prepared(const uint32_t *maskA, int64_t strideA, const void *preparedB,
                              size_t preparedB_bytes, int preparedB_format, int batch, int M, int N, int K, const void *s_a,
                              int a_scale_mode, const void *s_b, int b_scale_mode, float alpha,
                              void *out, int64_t ldo, int64_t stride_out, bwta_stream_t stream);

/*
 * Binary weights from full-precision ones (the paper's W_sign equation), per output channel n:
 *   mu_n = mean_k W[n, k];  wsign bit = 1 iff W[n, k] - mu_n < 0;  s_w[n] = fp16( mean_k |W[n, k] - mu_n| )
 * W is fp16 [N, ldw]; wsign is written in the layout of bwta_pack_weights; s_w is fp16 [N] (the
 * scale that minimises ||(W - mu) - s sign(W - mu)||^2; the printed (1/n)||W||_F is read as this
 * l1 mean).  Sums are exact (binary16 values are integers in units of 2^-24), so the planes equal
 * exact arithmetic bit for bit; the scale is rounded once from a double.  A NaN / Inf entry adds
 * nothing to either sum, while both means still divide by K (mu_n = finite sum / K; s_w[n] = sum
 * over the finite entries of |W - mu_n|, / K); its own bit is +Inf -> +1, -Inf and NaN -> -1.
 * K <= 32768.
 */
int bwta_prepare_weights(const void *W, int64_t ldw, int N, int K, uint32_t *wsign, void *s_w,
                         bwta_stream_t stream);

/*
 * The value the paper initialises the activation scale with (the s_A^0 equation), per token:
 *   s[m] = fp16( 2 * mean_k |A[m, k]| )   A fp16 [M, lda], s fp16 [M]; exact sum, one rounding;
 * NaN / Inf entries count as 0.  K <= 32768.
 */
int bwta_act_scale(const void *A, int64_t lda, int M, int K, void *s, bwta_stream_t stream);

/*
 * bwta_act_scale and bwta_prepare_act in one pass over A (the single-pass form of the same
 * s_A^0 equation followed by the ternary function): writes s_a[m] = fp16(2 * mean_k |A[m, k]|)
 * (fp16 [M], the same bits as bwta_act_scale) and ternarises every token with its own scale into
 * `prepared`, reporting the layout in *prepared_format (see bwta_prepare_act; pass s_a with
 * BWTA_SCALE_VECTOR to bwta_gemm_prepared).  A row whose scale comes out 0 (all zeros or
 * non-finite) ternarises to zero.  K <= 32768.
 */
int bwta_prepare_act_autoscale(const void *A, int64_t lda, int M, int K, void *s_a, void *prepared,
                               size_t prepared_bytes, int *prepared_format, bwta_stream_t stream);

/* Human-readable text for a return code (static storage). */
const char *bwta_strerror(int code);
/* hipError_t value behind the calling thread's most recent BWTA_ERR_HIP (0 if none). */
int bwta_last_hip_error(void);
/* Select the contraction kernel family (process-wide).  Returns BWTA_OK or UNSUPPORTED. */
int bwta_set_path(int path);
int bwta_get_path(void);
/* Library version, major * 100 + minor. */
int bwta_version(void);
/* A short hex digest of the sources this library was built from (static storage): lets a
 * measurement that was taken on one build be told apart from another build's. */
const char *bwta_build_id(void);

#ifdef __cplusplus
}
#endif
#endif /* BWTA_H */
