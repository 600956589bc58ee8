/*
 * CPU oracle for the BWTA (binary weights, ternary activations) linear layer.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the tests, the smoke
 * check and the benchmark's cpu_baseline leg may call it.  It shares no code,
 * header, table or helper with the HIP library and neither includes the other.
 *
 * Everything here is the plain definition, written out slowly:
 *   - fp16 values are decoded by hand from their bit fields into double;
 *   - ternarisation follows the paper's "Ternary Function" equation with exact
 *     real comparisons (a against +-0.5*s, both exact in double, no division);
 *   - weights follow the paper's "Binary Functions" sign equation;
 *   - the matrix product is a triple loop over unpacked int8 operands with an
 *     int32 accumulator (the BWTA linear-layer equation, "Basic Layers for
 *     Linear and MatMul");
 *   - bit planes use the paper's polarity (negative -> bit 1, positive -> bit 0,
 *     two planes for a ternary operand; "Instruction-level Parallel Bitpack" and
 *     "Comprehensive Computational Implementations");
 *   - three packed evaluations of the same product (mask/sign form, the
 *     xor-difference form behind the paper's "two xor + one sub" Case 1, and the
 *     four-AND form the paper spells out for Case 1) exist only so tests can
 *     check that they equal the triple loop;
 *   - the epilogue is s_W * s_A * acc evaluated exactly in double (the product
 *     of a 14-bit integer and two 11-bit significands fits in 53 bits) and
 *     rounded once, to nearest even, to fp16.
 *
 * Pins (tests marked "not gpu"): exhaustive fp16 decode/round against numpy,
 * exhaustive ternarisation of all 65536 fp16 patterns, brute force over every
 * operand pair for tiny K, equality of the four product forms, algebraic
 * invariants, the XNOR-popcount special case, and an independent numpy integer
 * matmul.  No function here is "parity unpinned".
 *
 * Loops over rows are split across OpenMP threads; nothing else is tuned.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_SCALE_NONE 0    /* every scale is 1.0, pointer ignored       */
#define ORACLE_SCALE_SCALAR 1  /* one fp16 value for the whole tensor       */
#define ORACLE_SCALE_VECTOR 2  /* one fp16 value per row (token / channel)  */

int bwta_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void bwta_oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ---- IEEE-754 binary16, by hand ------------------------------------------------ */

/* sign(1) exponent(5, bias 15) fraction(10).  Returns NaN for NaN patterns. */
double bwta_oracle_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (expo == 0) {
        v = ldexp((double)frac, -24);            /* zero and subnormals: frac * 2^-24 */
    } else if (expo == 31) {
        v = frac ? NAN : INFINITY;
    } else {
        v = ldexp((double)(1024 + frac), expo - 25); /* (1 + frac/1024) * 2^(expo-15) */
    }
    return sign ? -v : v;
}

/* Round a double to the nearest binary16 (ties to even), overflow -> +-Inf. */
uint16_t bwta_oracle_double_to_half(double x)
{
    uint16_t sign = 0;
    if (isnan(x)) return 0x7e00;
    if (signbit(x)) { sign = 0x8000; x = -x; }
    if (isinf(x)) return (uint16_t)(sign | 0x7c00);
    if (x == 0.0) return sign;
    int e;
    (void)frexp(x, &e);         /* x = m * 2^e, m in [0.5, 1)  ->  2^(e-1) <= x < 2^e */
    int expo = e - 1;           /* unbiased exponent of x */
    if (expo < -14) expo = -14; /* subnormal range shares the spacing of 2^-14 */
    double quantum = ldexp(1.0, expo - 10);
    /* x / quantum is exact (power of two); nearbyint rounds ties to even under the
       default rounding mode, which nothing in this file changes. */
    double n = nearbyint(x / quantum);
    if (n >= 2048.0) { n = 1024.0; expo += 1; quantum *= 2.0; } /* carried into next binade */
    if (expo > 15) return (uint16_t)(sign | 0x7c00);
    uint16_t bits;
    if (n < 1024.0) bits = (uint16_t)n;                              /* subnormal or zero */
    else bits = (uint16_t)(((expo + 15) << 10) | ((int)n - 1024));   /* normal */
    return (uint16_t)(sign | bits);
}

static double scale_value(const uint16_t *s, int mode, int64_t row)
{
    if (mode == ORACLE_SCALE_NONE || s == NULL) return 1.0;
    if (mode == ORACLE_SCALE_SCALAR) return bwta_oracle_half_to_double(s[0]);
    return bwta_oracle_half_to_double(s[row]);
}

/* ---- element definitions ------------------------------------------------------- */

/* Ternary Function: +1 if a/s >= 0.5, 0 if -0.5 <= a/s < 0.5, -1 if a/s < -0.5.
 * With s > 0 this is a >= 0.5*s / a < -0.5*s over the reals; both sides are exact
 * in double.  Reading for what the paper leaves open: a scale that is not a finite
 * positive number ternarises the row to 0; NaN activations satisfy no inequality
 * and give 0; +-Inf give +-1. */
int bwta_oracle_ternary_value(double a, double s)
{
    if (!(s > 0.0) || isinf(s)) return 0;
    if (isnan(a)) return 0;
    double half = 0.5 * s;
    if (a >= half) return 1;
    if (a < -half) return -1;
    return 0;
}

/* Binary Functions, sign: +1 if w >= 0, -1 otherwise (so -0.0 -> +1, NaN -> -1). */
int bwta_oracle_sign_value(double w)
{
    return (w >= 0.0) ? 1 : -1;
}

/* bool(a, s) for non-negative activations: 1 if a/s >= 0.5 else 0. */
int bwta_oracle_bool_value(double a, double s)
{
    if (!(s > 0.0) || isinf(s)) return 0;
    if (isnan(a)) return 0;
    return (a >= 0.5 * s) ? 1 : 0;
}

/* ---- tensor-level steps --------------------------------------------------------- */

/* A: fp16 bits [M, lda]; t: int8 [M, K] dense. */
void bwta_oracle_ternarize(const uint16_t *A, int64_t lda, const uint16_t *s_a, int scale_mode,
                           int M, int K, int8_t *t)
{
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        double s = scale_value(s_a, scale_mode, m);
        for (int k = 0; k < K; ++k) {
            double a = bwta_oracle_half_to_double(A[(int64_t)m * lda + k]);
            t[(int64_t)m * K + k] = (int8_t)bwta_oracle_ternary_value(a, s);
        }
    }
}

/* W: fp16 bits [N, ldw]; w: int8 [N, K] dense, values +-1. */
void bwta_oracle_sign_weights(const uint16_t *W, int64_t ldw, int N, int K, int8_t *w)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            w[(int64_t)n * K + k] =
                (int8_t)bwta_oracle_sign_value(bwta_oracle_half_to_double(W[(int64_t)n * ldw + k]));
}

/* Words per packed row: rows are padded with zero bits to a multiple of 128 bits. */
int64_t bwta_oracle_row_words(int K)
{
    return 4 * (((int64_t)K + 127) / 128);
}

/* Two planes for a ternary operand.  Element k sits in word k/32 at bit k%32
 * (least significant bit first).  mask bit = (t != 0); sign bit = (t < 0), so the
 * paper's A- plane is `sign` and its A+ plane is `mask ^ sign`; a zero has both
 * bits clear.  nnz[m] (optional) = number of nonzero elements of row m. */
void bwta_oracle_pack_act(const int8_t *t, int M, int K, uint32_t *mask, uint32_t *sign,
                          int32_t *nnz)
{
    int64_t rw = bwta_oracle_row_words(K);
    for (int m = 0; m < M; ++m) {
        int32_t count = 0;
        for (int64_t w = 0; w < rw; ++w) { mask[m * rw + w] = 0; sign[m * rw + w] = 0; }
        for (int k = 0; k < K; ++k) {
            int v = t[(int64_t)m * K + k];
            if (v != 0) { mask[m * rw + k / 32] |= (uint32_t)1 << (k % 32); ++count; }
            if (v < 0) sign[m * rw + k / 32] |= (uint32_t)1 << (k % 32);
        }
        if (nnz) nnz[m] = count;
    }
}

/* One plane for a binary operand: bit = 1 iff w is negative. */
void bwta_oracle_pack_weights(const int8_t *w, int N, int K, uint32_t *wsign)
{
    int64_t rw = bwta_oracle_row_words(K);
    for (int n = 0; n < N; ++n) {
        for (int64_t q = 0; q < rw; ++q) wsign[n * rw + q] = 0;
        for (int k = 0; k < K; ++k)
            if (w[(int64_t)n * K + k] < 0) wsign[n * rw + k / 32] |= (uint32_t)1 << (k % 32);
    }
}

/* Inverse of the two packers (used by round-trip tests). */
void bwta_oracle_unpack_act(const uint32_t *mask, const uint32_t *sign, int M, int K, int8_t *t)
{
    int64_t rw = bwta_oracle_row_words(K);
    for (int m = 0; m < M; ++m)
        for (int k = 0; k < K; ++k) {
            int nz = (mask[m * rw + k / 32] >> (k % 32)) & 1;
            int ng = (sign[m * rw + k / 32] >> (k % 32)) & 1;
            t[(int64_t)m * K + k] = (int8_t)(nz ? (ng ? -1 : 1) : 0);
        }
}

void bwta_oracle_unpack_weights(const uint32_t *wsign, int N, int K, int8_t *w)
{
    int64_t rw = bwta_oracle_row_words(K);
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            w[(int64_t)n * K + k] = (int8_t)(((wsign[n * rw + k / 32] >> (k % 32)) & 1) ? -1 : 1);
}

/* acc[m, n] = sum_k t[m, k] * w[n, k]  -- the definition, int32 accumulator.
 * Output orientation is [M, N]: the paper writes W (x) A^T, the same numbers transposed. */
void bwta_oracle_gemm_unpacked(const int8_t *t, const int8_t *w, int M, int N, int K, int32_t *acc)
{
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m)
        for (int n = 0; n < N; ++n) {
            int32_t sum = 0;
            for (int k = 0; k < K; ++k)
                sum += (int32_t)t[(int64_t)m * K + k] * (int32_t)w[(int64_t)n * K + k];
            acc[(int64_t)m * N + n] = sum;
        }
}

static int count_bits(uint32_t x)
{
    int c = 0;
    while (x) { c += (int)(x & 1u); x >>= 1; }
    return c;
}

/* The same product from packed planes, three ways (form 0, 1, 2):
 *   0: popc(mask) - 2 popc(mask & (sign ^ wsign))
 *   1: popc(wsign ^ A+) - popc(wsign ^ A-)          (two xor-popcounts and one subtraction)
 *   2: -popc(W & A+) + popc(W & A-) + popc(~W & A+) - popc(~W & A-)   (four and-popcounts)
 * with A- = sign, A+ = mask ^ sign, W = wsign.  In form 1 the popc(W) terms cancel,
 * which is why padding bits cancel too; in form 2 the complement of W is masked by A+/A-.
 * These exist for invariants only; the definition is bwta_oracle_gemm_unpacked. */
void bwta_oracle_gemm_packed(int form, const uint32_t *mask, const uint32_t *sign,
                             const uint32_t *wsign, int M, int N, int K, int32_t *acc)
{
    int64_t rw = bwta_oracle_row_words(K);
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m)
        for (int n = 0; n < N; ++n) {
            int32_t sum = 0;
            for (int64_t q = 0; q < rw; ++q) {
                uint32_t mk = mask[m * rw + q], sg = sign[m * rw + q], W = wsign[n * rw + q];
                uint32_t aneg = sg, apos = mk ^ sg;
                if (form == 0) {
                    sum += count_bits(mk) - 2 * count_bits(mk & (sg ^ W));
                } else if (form == 1) {
                    sum += count_bits(W ^ apos) - count_bits(W ^ aneg);
                } else {
                    sum += -count_bits(W & apos) + count_bits(W & aneg) + count_bits(~W & apos) -
                           count_bits(~W & aneg);
                }
            }
            acc[(int64_t)m * N + n] = sum;
        }
}

/* out[m, n] = fp16( s_w[n] * s_a[m] * acc[m, n] ), the prefix of the BWTA linear
 * equation, evaluated exactly and rounded once (nearest even).  out: fp16 bits [M, ldo]. */
void bwta_oracle_epilogue(const int32_t *acc, const uint16_t *s_a, int a_mode, const uint16_t *s_w,
                          int w_mode, int M, int N, uint16_t *out, int64_t ldo)
{
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        double sa = scale_value(s_a, a_mode, m);
        for (int n = 0; n < N; ++n) {
            double sw = scale_value(s_w, w_mode, n);
            double v = ((double)acc[(int64_t)m * N + n] * sa) * sw;
            out[(int64_t)m * ldo + n] = bwta_oracle_double_to_half(v);
        }
    }
}

/* ---- attention MatMuls ("Basic Layers for Linear and MatMul": BWTA_QK and BWTA_Att) ------- */

/* A: fp16 bits [M, lda] -> b int8 [M, K] in {0, 1} by the bool function. */
void bwta_oracle_boolize(const uint16_t *A, int64_t lda, const uint16_t *s_a, int scale_mode, int M, int K,
                         int8_t *b)
{
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        double s = scale_value(s_a, scale_mode, m);
        for (int k = 0; k < K; ++k)
            b[(int64_t)m * K + k] = (int8_t)bwta_oracle_bool_value(bwta_oracle_half_to_double(A[m * lda + k]), s);
    }
}

/* Packed evaluations of a[m,:] . b[n,:] for two operands given as (mask, sign) planes; a sign
 * pointer may be NULL (boolean operand).  form 0: the four-AND expression of arithmetic Case 3,
 * popc(A+ & B+) + popc(A- & B-) - popc(A+ & B-) - popc(A- & B+); with A- = 0 it is Case 2,
 * popc(Att & V+) - popc(Att & V-).  form 1: popc(u) - 2 popc(u & (sA ^ sB)), u = maskA & maskB.
 * For invariants only; the definition is bwta_oracle_gemm_unpacked on the unpacked operands. */
void bwta_oracle_matmul_tt_packed(int form, const uint32_t *maskA, const uint32_t *signA, const uint32_t *maskB,
                                  const uint32_t *signB, int M, int N, int K, int32_t *acc)
{
    int64_t rw = bwta_oracle_row_words(K);
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m)
        for (int n = 0; n < N; ++n) {
            int32_t sum = 0;
            for (int64_t q = 0; q < rw; ++q) {
                uint32_t ma = maskA[m * rw + q], sa = signA ? signA[m * rw + q] & ma : 0u;
                uint32_t mb = maskB[n * rw + q], sb = signB ? signB[n * rw + q] & mb : 0u;
                if (form == 0) {
                    uint32_t ap = ma ^ sa, an = sa, bp = mb ^ sb, bn = sb;
                    sum += count_bits(ap & bp) + count_bits(an & bn) - count_bits(ap & bn) - count_bits(an & bp);
                } else {
                    uint32_t u = ma & mb;
                    sum += count_bits(u) - 2 * count_bits(u & (sa ^ sb));
                }
            }
            acc[(int64_t)m * N + n] = sum;
        }
}

/* out[m, n] = fp16( acc[m, n] * s ),  s = fp32( alpha * (s_a[m] * s_b[n]) ): the scale prefix of the
 * BWTA_QK rule (alpha = 1/sqrt(D), given as an fp32 number) and of the BWTA_Att rule (alpha = 1).
 * s_a * s_b is exact (two 11-bit significands); the product with alpha is formed exactly in double
 * (24 + 22 bits) and rounded once to fp32; acc * s is exact in double and rounded once to fp16. */
void bwta_oracle_epilogue_alpha(const int32_t *acc, const uint16_t *s_a, int a_mode, const uint16_t *s_b,
                                int b_mode, float alpha, int M, int N, uint16_t *out, int64_t ldo)
{
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        double sa = scale_value(s_a, a_mode, m);
        for (int n = 0; n < N; ++n) {
            double sb = scale_value(s_b, b_mode, n);
            float s = (float)((double)alpha * (sa * sb));
            out[(int64_t)m * ldo + n] = bwta_oracle_double_to_half((double)acc[(int64_t)m * N + n] * (double)s);
        }
    }
}

/* ---- weight preparation and the activation scale's starting value ------------------------- */

/* A finite binary16 value as an integer count of 2^-24 (exact); 0 for NaN / Inf. */
static int64_t half_fixed(uint16_t h, int *finite)
{
    int sign = (h >> 15) & 1, expo = (h >> 10) & 0x1f, frac = h & 0x3ff;
    int64_t v;
    *finite = expo != 31;
    if (expo == 31) return 0;
    v = expo == 0 ? (int64_t)frac : ((int64_t)(1024 + frac) << (expo - 1));
    return sign ? -v : v;
}

/* num / den (den > 0) rounded once to binary16, ties to even, by integer arithmetic only. */
static uint16_t ratio_to_half(unsigned __int128 num, unsigned __int128 den)
{
    if (num == 0) return 0;
    int e = 16; /* largest e with 2^e <= num / den, searched downwards; values >= 2^16 overflow */
    if (num >= (den << 16)) return 0x7c00;
    while (e > -25) {
        --e;
        if (e >= 0 ? num >= (den << e) : (num << -e) >= den) break;
    }
    int qe = (e < -14 ? -14 : e) - 10; /* exponent of the spacing of binary16 numbers at this magnitude */
    unsigned __int128 n2 = qe >= 0 ? num : num << -qe, d2 = qe >= 0 ? den << qe : den;
    unsigned __int128 q = n2 / d2, r = n2 - q * d2;
    if (2 * r > d2 || (2 * r == d2 && (q & 1))) ++q;
    int expo = e < -14 ? -14 : e;
    if (q >= 2048) { q = 1024; ++expo; }
    if (expo > 15) return 0x7c00;
    if (q < 1024) return (uint16_t)q; /* subnormal (or rounded up to the smallest normal: bits 0x400) */
    return (uint16_t)(((expo + 15) << 10) | ((int)q - 1024));
}

/* Binary weights from full-precision ones (the W_sign equation): per output channel n,
 *   mu_n = mean_k W[n, k],  w[n, k] = sign(W[n, k] - mu_n),  s_w[n] = mean_k |W[n, k] - mu_n|
 * (the scale that minimises || (W - mu) - s sign(W - mu) ||^2; the printed (1/n)||W||_F is read as
 * this l1 mean).  All decisions are exact: binary16 values are integers in units of 2^-24, so
 * W[n,k] - mu_n >= 0 is the integer test K * W >= sum(W).  A non-finite entry adds nothing
 * to either sum while both means still divide by K (mu_n = finite sum / K, s_w[n] = sum over the
 * finite entries of |W - mu_n|, / K); its own sign is +Inf -> +1, -Inf and NaN -> -1.  w: int8 [N, K]; s_w: fp16 bits [N]. */
void bwta_oracle_prepare_weights(const uint16_t *W, int64_t ldw, int N, int K, int8_t *w, uint16_t *s_w)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        const uint16_t *row = W + (int64_t)n * ldw;
        int64_t S = 0;
        int fin;
        for (int k = 0; k < K; ++k) S += half_fixed(row[k], &fin);
        unsigned __int128 T = 0;
        for (int k = 0; k < K; ++k) {
            int64_t v = half_fixed(row[k], &fin);
            if (!fin) {
                w[(int64_t)n * K + k] = (row[k] == 0x7c00) ? 1 : -1;
                continue;
            }
            __int128 d = (__int128)v * K - S;
            w[(int64_t)n * K + k] = d >= 0 ? 1 : -1;
            T += (unsigned __int128)(d >= 0 ? d : -d);
        }
        s_w[n] = ratio_to_half(T, ((unsigned __int128)K * K) << 24);
    }
}

/* The value the activation scale starts from (the s_A^0 equation), per token:
 *   s[m] = 2 * mean_k |A[m, k]|, exact sum, rounded once to binary16.  Non-finite entries count as 0. */
void bwta_oracle_act_scale(const uint16_t *A, int64_t lda, int M, int K, uint16_t *s)
{
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        unsigned __int128 T = 0;
        int fin;
        for (int k = 0; k < K; ++k) {
            int64_t v = half_fixed(A[(int64_t)m * lda + k], &fin);
            T += (unsigned __int128)(v >= 0 ? v : -v);
        }
        s[m] = ratio_to_half(2 * T, (unsigned __int128)K << 24);
    }
}

/* The whole layer on fp16 activations and unpacked +-1 weights:
 * ternarise -> triple-loop product -> scale epilogue.  t_out/acc_out may be NULL. */
void bwta_oracle_linear(const uint16_t *A, int64_t lda, const uint16_t *s_a, int a_mode,
                        const int8_t *w, const uint16_t *s_w, int w_mode, int M, int N, int K,
                        int8_t *t_scratch, int32_t *acc_scratch, uint16_t *out, int64_t ldo)
{
    bwta_oracle_ternarize(A, lda, s_a, a_mode, M, K, t_scratch);
    bwta_oracle_gemm_unpacked(t_scratch, w, M, N, K, acc_scratch);
    bwta_oracle_epilogue(acc_scratch, s_a, a_mode, s_w, w_mode, M, N, out, ldo);
}
