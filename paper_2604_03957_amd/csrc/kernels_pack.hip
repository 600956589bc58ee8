// Ternarise + bit-pack activations, sign-pack weights (paper: "Ternary Function" and sign
// equations; "Instruction-level Parallel Bitpack").  Bandwidth-bound streaming kernels: every
// lane takes 8 consecutive elements with one 128-bit (fp16) or 64-bit (int8) load, turns them
// into one byte per plane, and the four lanes of a quad assemble a 32-bit plane word.
#include "bwta_internal.h"

namespace bwta {

namespace {

constexpr int kThreads = 256;
// four groups per thread only when that still leaves a few workgroups per compute unit
constexpr int64_t kQuadGroupMinThreads = 1024 * kThreads;

// OR a per-lane byte into its quad's 32-bit word (lane q of the quad supplies byte q).
__device__ __forceinline__ uint32_t quad_word(uint32_t byte, int lane)
{
    uint32_t v = byte << (8 * (lane & 3));
    v |= __shfl_xor(v, 1);
    v |= __shfl_xor(v, 2);
    return v;
}

struct TernaryBits {
    uint32_t nz, neg;
};

// 8 fp16 values against the exact thresholds +-h (h = 0.5 * s in fp32, exact).
__device__ __forceinline__ TernaryBits ternary_bits_fp16(const uint16_t v[8], int nvalid, float h, bool ok)
{
    TernaryBits r{0u, 0u};
    // an invalid scale becomes a NaN threshold (every compare fails); elements past nvalid were
    // loaded as +0 and fail both compares too, h being positive
    (void)nvalid;
    const float hp = ok ? h : __builtin_nanf(""), hn = -hp;
    uint32_t both = 0;  // bits 0..7 non-zero flags, bits 8..15 negative flags
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float a = half_bits_to_float(v[i]);
        uint32_t sel = a >= hp ? 1u : 0u;  // NaN fails both compares
        sel = a < hn ? 0x101u : sel;
        both = (sel << i) | both;
    }
    r.nz = both & 0xffu;
    r.neg = both >> 8;
    return r;
}

template <int DTYPE>  // 0 = fp16 -> ternary, 1 = int8 ternary, 2 = fp16 -> boolean (the bool function: 1 iff a >= 0.5 s)
__global__ __launch_bounds__(kThreads) void k_quantize_pack(const void *__restrict__ A, int64_t lda,
                                                            ScaleArg s_a, int M, int K, int rw,
                                                            uint32_t *__restrict__ mask,
                                                            uint32_t *__restrict__ sign, int vec_ok)
{
    const int c8 = rw * 4;  // byte-groups (8 elements) per packed row, a multiple of 16
    const int64_t total = (int64_t)M * c8;
    const int64_t gid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (gid >= total) return;  // whole quads leave together (total % 4 == 0)
    const int m = (int)(gid / c8);
    const int c = (int)(gid - (int64_t)m * c8);
    const int k0 = c * 8;
    const int nvalid = K - k0 >= 8 ? 8 : (K - k0 > 0 ? K - k0 : 0);
    TernaryBits tb{0u, 0u};
    if (DTYPE == 0 || DTYPE == 2) {
        // the scale is requested before the data and by every lane (without a scale: a dropped read
        // of the first element), so the two requests share one memory round trip
        const bool have_scale = s_a.mode != 0 && s_a.ptr != nullptr;
        const uint16_t s_bits = *(have_scale ? s_a.ptr + (s_a.mode == 1 ? 0 : m) : (const uint16_t *)A);
        const uint16_t *row = (const uint16_t *)A + (int64_t)m * lda;
        uint16_t v[8];
        if (nvalid == 8 && vec_ok) {
            uint4 q = *(const uint4 *)(row + k0);
            v[0] = q.x & 0xffff; v[1] = q.x >> 16; v[2] = q.y & 0xffff; v[3] = q.y >> 16;
            v[4] = q.z & 0xffff; v[5] = q.z >> 16; v[6] = q.w & 0xffff; v[7] = q.w >> 16;
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = i < nvalid ? row[k0 + i] : (uint16_t)0;
        }
        const float s = have_scale ? half_bits_to_float(s_bits) : 1.0f;
        const bool ok = (s > 0.0f) && (s < __builtin_inff());
        tb = ternary_bits_fp16(v, nvalid, 0.5f * s, ok);
        if (DTYPE == 2) tb.nz &= ~tb.neg;  // boolean: only a >= 0.5 s counts, and there is no sign plane
    } else {
        const int8_t *row = (const int8_t *)A + (int64_t)m * lda;
        int8_t v[8];
        if (nvalid == 8 && vec_ok) {
            uint2 q = *(const uint2 *)(row + k0);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                v[i] = (int8_t)(q.x >> (8 * i));
                v[4 + i] = (int8_t)(q.y >> (8 * i));
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = i < nvalid ? row[k0 + i] : (int8_t)0;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            tb.nz |= (uint32_t)(v[i] != 0) << i;
            tb.neg |= (uint32_t)(v[i] < 0) << i;
        }
    }
    const int lane = threadIdx.x & 63;
    uint32_t wm = quad_word(tb.nz, lane);
    uint32_t ws = quad_word(tb.neg, lane);
    const int64_t widx = (int64_t)m * rw + (c >> 2);
    if ((lane & 3) == 0) mask[widx] = wm;
    if (DTYPE != 2 && (lane & 3) == 1) sign[widx] = ws;
}

// The same operation for 16-byte aligned fp16 rows whose K is a multiple of 8 (every group of 8 is
// whole or entirely padding): a thread takes four groups of one row, a quarter row apart, and
// issues its scale request and all four 128-bit loads before anything is used, so four times the
// bytes are in flight per wavefront.  Index space: row m, word w0 in the first quarter of the row,
// quad lane q; group u is byte-group 4 (w0 + u rw / 4) + q.
template <int DTYPE>  // 0 = ternary, 2 = boolean
__global__ __launch_bounds__(kThreads) void k_quantize_pack_vec(const uint16_t *__restrict__ A, int64_t lda,
                                                                ScaleArg s_a, int M, int K, int rw,
                                                                uint32_t *__restrict__ mask,
                                                                uint32_t *__restrict__ sign)
{
    const int64_t total = (int64_t)M * rw;  // threads with work: M rows x rw / 4 words x 4 lanes
    const int64_t gid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const bool live = gid < total;  // whole quads together (rw % 4 == 0)
    const int64_t gc = live ? gid : 0;
    const int m = (int)(gc / rw), rem = (int)(gc - (int64_t)m * rw);
    const int w0 = rem >> 2, q = rem & 3, qw = rw >> 2;
    const bool have_scale = s_a.mode != 0 && s_a.ptr != nullptr;
    const uint16_t s_bits = *(have_scale ? s_a.ptr + (s_a.mode == 1 ? 0 : m) : A);
    const uint16_t *row = A + (int64_t)m * lda;
    uint4 x[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int k0 = 8 * (4 * (w0 + u * qw) + q);
        x[u] = *(const uint4 *)(k0 < K ? row + k0 : A);  // padding groups re-read the first bytes and drop them
    }
    __builtin_amdgcn_sched_barrier(0);
    const float s = have_scale ? half_bits_to_float(s_bits) : 1.0f;
    const bool ok = (s > 0.0f) && (s < __builtin_inff());
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int w = w0 + u * qw, k0 = 8 * (4 * w + q);
        const uint4 xv = k0 < K ? x[u] : make_uint4(0, 0, 0, 0);
        const uint16_t v[8] = {(uint16_t)xv.x, (uint16_t)(xv.x >> 16), (uint16_t)xv.y, (uint16_t)(xv.y >> 16),
                               (uint16_t)xv.z, (uint16_t)(xv.z >> 16), (uint16_t)xv.w, (uint16_t)(xv.w >> 16)};
        TernaryBits tb = ternary_bits_fp16(v, 8, 0.5f * s, ok);
        if (DTYPE == 2) tb.nz &= ~tb.neg;
        const uint32_t wm = quad_word(tb.nz, lane);
        const uint32_t ws = DTYPE == 2 ? 0u : quad_word(tb.neg, lane);
        const int64_t widx = (int64_t)m * rw + w;
        if (live && q == 0) mask[widx] = wm;
        if (DTYPE != 2 && live && q == 1) sign[widx] = ws;
    }
}

template <int DTYPE>
__global__ __launch_bounds__(kThreads) void k_pack_weights(const void *__restrict__ W, int64_t ldw,
                                                           int N, int K, int rw,
                                                           uint32_t *__restrict__ wsign, int vec_ok)
{
    const int c8 = rw * 4;
    const int64_t total = (int64_t)N * c8;
    const int64_t gid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (gid >= total) return;
    const int n = (int)(gid / c8);
    const int c = (int)(gid - (int64_t)n * c8);
    const int k0 = c * 8;
    const int nvalid = K - k0 >= 8 ? 8 : (K - k0 > 0 ? K - k0 : 0);
    uint32_t bits = 0;
    if (DTYPE == 0) {
        const uint16_t *row = (const uint16_t *)W + (int64_t)n * ldw;
        uint16_t v[8];
        if (nvalid == 8 && vec_ok) {
            uint4 q = *(const uint4 *)(row + k0);
            v[0] = q.x & 0xffff; v[1] = q.x >> 16; v[2] = q.y & 0xffff; v[3] = q.y >> 16;
            v[4] = q.z & 0xffff; v[5] = q.z >> 16; v[6] = q.w & 0xffff; v[7] = q.w >> 16;
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = i < nvalid ? row[k0 + i] : (uint16_t)0;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float w = half_bits_to_float(v[i]);
            bits |= (uint32_t)((i < nvalid) && !(w >= 0.0f)) << i;  // "otherwise" includes NaN
        }
    } else {
        const int8_t *row = (const int8_t *)W + (int64_t)n * ldw;
        if (nvalid == 8 && vec_ok) {
            uint2 q = *(const uint2 *)(row + k0);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                bits |= ((q.x >> (8 * i + 7)) & 1u) << i;
                bits |= ((q.y >> (8 * i + 7)) & 1u) << (4 + i);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                int8_t w = i < nvalid ? row[k0 + i] : (int8_t)0;
                bits |= (uint32_t)(w < 0) << i;
            }
        }
    }
    const int lane = threadIdx.x & 63;
    uint32_t word = quad_word(bits, lane);
    if ((lane & 3) == 0) wsign[(int64_t)n * rw + (c >> 2)] = word;
}

// nnz[m] = popcount of mask row m; one wavefront per row.
__global__ __launch_bounds__(kThreads) void k_row_popcount(const uint32_t *__restrict__ mask, int M,
                                                           int rw, int32_t *__restrict__ nnz)
{
    const int lane = threadIdx.x & 63;
    const int m = blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (m >= M) return;
    int c = 0;
    for (int w = lane; w < rw; w += 64) c += __popc(mask[(int64_t)m * rw + w]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) c += __shfl_xor(c, off);
    if (lane == 0) nnz[m] = c;
}

// ---- weight preparation from full-precision weights, and the activation scale's starting value ----
//
// Binary16 values are integers in units of 2^-24 (|v| < 2^40), so a row's sum is an exact 64-bit
// integer whatever the order of the additions, and "W[n,k] - mean >= 0" is the integer test
// K * W[n,k] >= sum.  Every discrete decision is therefore identical to exact arithmetic.

// non-negative double -> binary16 bits, round to nearest even, straight from the 53-bit significand
// (going through fp32 would round twice)
__device__ __forceinline__ uint16_t double_to_half_bits(double x)
{
    if (!(x > 0.0)) return 0;
    const unsigned long long b = (unsigned long long)__double_as_longlong(x);
    int e = (int)((b >> 52) & 0x7ff) - 1023;
    if (e > 15) return 0x7c00;
    if (e < -26) return 0;  // below half of the smallest subnormal
    const unsigned long long mant = (b & ((1ull << 52) - 1)) | (1ull << 52);
    const int shift = 42 + (e < -14 ? -14 - e : 0);  // bits dropped: keep 11 (normal) or fewer (subnormal)
    unsigned long long q = mant >> shift;
    const unsigned long long rem = mant & ((1ull << shift) - 1), half = 1ull << (shift - 1);
    if (rem > half || (rem == half && (q & 1))) ++q;
    if (e < -14) return (uint16_t)q;  // subnormal, or exactly the smallest normal (q = 1024)
    if (q == 2048) {
        q = 1024;
        ++e;
    }
    if (e > 15) return 0x7c00;
    return (uint16_t)(((e + 15) << 10) | (int)(q - 1024));
}

template <int NT, typename T>
__device__ __forceinline__ T block_sum(T v, T *scratch /* [NT / 64] */)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    __syncthreads();  // scratch may still be read from a previous call
    if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
    __syncthreads();
    T r = scratch[0];
#pragma unroll
    for (int i = 1; i < NT / 64; ++i) r += scratch[i];
    return r;
}

__device__ __forceinline__ void load8_halfs(const uint16_t *row, int k0, int nvalid, bool vec_ok, uint16_t v[8])
{
    if (nvalid == 8 && vec_ok) {
        const uint4 q = *(const uint4 *)(row + k0);
        v[0] = q.x & 0xffff; v[1] = q.x >> 16; v[2] = q.y & 0xffff; v[3] = q.y >> 16;
        v[4] = q.z & 0xffff; v[5] = q.z >> 16; v[6] = q.w & 0xffff; v[7] = q.w >> 16;
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = i < nvalid ? row[k0 + i] : (uint16_t)0;
    }
}

// two sums at once (one pair of barriers); every thread gets both
template <int NT>
__device__ __forceinline__ void block_sum2(long long &a, long long &b, long long *scratch /* [2 * NT / 64] */)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        a += __shfl_xor(a, off);
        b += __shfl_xor(b, off);
    }
    __syncthreads();  // scratch may still be read from a previous call
    if ((threadIdx.x & 63) == 0) {
        scratch[2 * (threadIdx.x >> 6)] = a;
        scratch[2 * (threadIdx.x >> 6) + 1] = b;
    }
    __syncthreads();
    a = scratch[0], b = scratch[1];
#pragma unroll
    for (int i = 1; i < NT / 64; ++i) a += scratch[2 * i], b += scratch[2 * i + 1];
}

// The row of a workgroup of NT threads, 8 halfs per 128-bit register, NG registers per thread (group g
// of thread t is byte-group t + NT g).  Few, long-lived wavefronts per row: the reductions, the
// division and the bound are a fixed cost per wavefront that dwarfs the per-element work.  All requests go out before the first value is used; the second
// pass of the weight preparation reads the registers, not memory.  Padding and out-of-row groups
// read as +0 (and are kept out of every count by nvalid).
template <int NG, int NT>
__device__ __forceinline__ void load_row_groups(const uint16_t *row, int K, int c8, bool whole, uint4 (&x)[NG])
{
    if (whole) {  // 16-byte aligned rows, K a multiple of 8: every group is whole or absent
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            const int k0 = 8 * ((int)threadIdx.x + NT * g);
            x[g] = *(const uint4 *)(k0 < K ? row + k0 : row);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int g = 0; g < NG; ++g)
            if (8 * ((int)threadIdx.x + NT * g) >= K) x[g] = make_uint4(0, 0, 0, 0);
    } else {
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            const int c = (int)threadIdx.x + NT * g, k0 = 8 * c;
            const int nvalid = c < c8 ? (K - k0 >= 8 ? 8 : (K - k0 > 0 ? K - k0 : 0)) : 0;
            uint16_t v[8];
            load8_halfs(row, k0, nvalid, false, v);
            x[g] = make_uint4(v[0] | ((uint32_t)v[1] << 16), v[2] | ((uint32_t)v[3] << 16),
                              v[4] | ((uint32_t)v[5] << 16), v[6] | ((uint32_t)v[7] << 16));
        }
    }
}

__device__ __forceinline__ uint16_t half_of(const uint4 &q, int i)
{
    const uint32_t w = i < 2 ? q.x : (i < 4 ? q.y : (i < 6 ? q.z : q.w));
    return (uint16_t)(w >> (16 * (i & 1)));
}

// A per-thread sum of at most 128 finite binary16 values is a multiple of 2^-24 below 2^23: exact
// in a double whatever the order.  This turns it into the integer count of 2^-24.
__device__ __forceinline__ long long double_units(double s) { return (long long)(s * 16777216.0); }

// The smallest value on the binary16 grid that is >= c * 2^-24 (c an integer count of 2^-24), as a
// float; +Inf if there is none.  For every finite binary16 x with integer count X:
// X >= c  <=>  float(x) >= result, so a 64-bit comparison per element becomes one float compare.
__device__ __forceinline__ float half_grid_ceil(long long c)
{
    const long long top = 65504ll << 24;
    if (c > top) return __builtin_inff();
    const bool negative = c < 0;
    unsigned long long a = (unsigned long long)(negative ? -c : c);
    if (a > (unsigned long long)top) a = (unsigned long long)top;  // only for c < -top: every finite x is >= c
    const int p = 63 - __builtin_clzll(a | 1ull);                   // position of the leading one
    if (p > 10) {  // grid spacing 2^(p-10): magnitudes round down for a negative bound, up for a positive one
        const unsigned long long sp = 1ull << (p - 10);
        a = negative ? (a & ~(sp - 1)) : ((a + sp - 1) & ~(sp - 1));
    }
    const float v = (float)(long long)a * 5.9604644775390625e-08f;  // at most 12 significant bits: exact
    return negative ? -v : v;
}

// One workgroup per output channel: mean (exact), sign(W - mean) packed like bwta_pack_weights,
// s_w = mean |W - mean|.  With X the integer count of 2^-24 of an element and S the row's exact sum,
// "W - mean < 0" is X K < S, i.e. X < ceil(S / K): one float compare against the bound above.  The
// sum of |X K - S| over the finite elements equals K (S - 2 Sn) - S (n - 2 nn) with Sn, nn the sum
// and count of the finite elements below the mean and n the count of finite elements, so the second
// pass needs only exact per-thread sums again; the final combination is done in double (one
// division, one rounding to binary16).
template <int NG, int NT>
__global__ __launch_bounds__(NT) void k_prepare_weights(const uint16_t *__restrict__ W, int64_t ldw, int K,
                                                              int rw, uint32_t *__restrict__ wsign,
                                                              uint16_t *__restrict__ s_w, int whole)
{
    __shared__ long long s_ll[2 * NT / 64];
    __shared__ float s_bound;
    const int n = blockIdx.x, c8 = rw * 4, lane = threadIdx.x & 63;
    uint4 x[NG];
    load_row_groups<NG, NT>(W + (int64_t)n * ldw, K, c8, whole != 0, x);

    double part = 0.0;
    int nfin = 0;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {  // elements past K were loaded as +0: finite, and they add nothing
            const uint16_t h = half_of(x[g], i);
            const bool fin = (h & 0x7c00) != 0x7c00;
            part += (double)(fin ? half_bits_to_float(h) : 0.0f);
            nfin += fin ? 0 : 1;  // counts the non-finite ones
        }
    }
    long long S = double_units(part), NF = nfin;
    block_sum2<NT>(S, NF, s_ll);
    NF = K - NF;  // finite elements of the row
    if (threadIdx.x == 0) {  // one 64-bit division per row, not per wavefront
        const long long q = S / K, r = S - q * K;
        s_bound = half_grid_ceil(q + (r > 0 ? 1 : 0));  // ceil(S / K)
    }
    __syncthreads();
    const float bound = s_bound;
    // The second pass recomputes its per-element predicates from the registers: kept opaque here,
    // or the compiler carries 64 of them per thread across the barriers in spilled scalar registers.
#pragma unroll
    for (int g = 0; g < NG; ++g) asm volatile("" : "+v"(x[g].x), "+v"(x[g].y), "+v"(x[g].z), "+v"(x[g].w));

    double below = 0.0;
    int nbelow = 0;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        const int c = (int)threadIdx.x + NT * g, k0 = 8 * c;
        uint32_t bits = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint16_t h = half_of(x[g], i);
            const float f = half_bits_to_float(h);
            const bool inside = k0 + i < K;
            const bool neg = inside && !(f >= bound);  // NaN and -Inf -> -1, +Inf -> +1
            const bool fin_neg = neg && (h & 0x7c00) != 0x7c00;
            bits |= (uint32_t)neg << i;
            below += (double)(fin_neg ? f : 0.0f);
            nbelow += fin_neg ? 1 : 0;
        }
        const uint32_t word = quad_word(bits, lane);  // whole quads stay together: c8 is a multiple of 4
        if (c < c8 && (lane & 3) == 0) wsign[(int64_t)n * rw + (c >> 2)] = word;
    }
    long long SN = double_units(below), NN = nbelow;
    block_sum2<NT>(SN, NN, s_ll);
    if (threadIdx.x == 0) {
        const double T = (double)K * (double)(S - 2 * SN) - (double)S * (double)(NF - 2 * NN);
        s_w[n] = double_to_half_bits(T / ((double)K * (double)K * 16777216.0));
    }
}

// One workgroup per token: s[m] = 2 * mean_k |A[m, k]| (exact integer sum, one division, one rounding).
template <int NG, int NT>
__global__ __launch_bounds__(NT) void k_act_scale(const uint16_t *__restrict__ A, int64_t lda, int K,
                                                        uint16_t *__restrict__ s, int whole)
{
    __shared__ long long s_ll[NT / 64];
    const int m = blockIdx.x, c8 = (K + 7) / 8;
    uint4 x[NG];
    load_row_groups<NG, NT>(A + (int64_t)m * lda, K, c8, whole != 0, x);
    double part = 0.0;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {  // elements past K were loaded as +0 and add nothing
            const uint16_t h = half_of(x[g], i) & 0x7fff;
            const float f = h < 0x7c00 ? half_bits_to_float(h) : 0.0f;  // NaN / Inf stay out
            part += (double)f;
        }
    }
    const long long S = block_sum<NT>(double_units(part), s_ll);
    if (threadIdx.x == 0) s[m] = double_to_half_bits((double)S / ((double)K * 8388608.0));  // 2 S / (K 2^24)
}

// The same scale and, from the same registers, the ternarised row: one pass over A where
// bwta_act_scale followed by bwta_prepare_act makes two.  FRAG: E2M1 fragments for the tiled
// matrix-core kernel (the grid also covers the padding rows of the last row blocks, and the threads
// the padding k steps: they write the zeros the product relies on); otherwise the two bit planes.
// Thread t's group g is elements 8 (t + NT g) ..: the four lanes of a hardware quad hold one
// 32-element plane word, which both output forms assemble inside the quad.
template <int NG, int NT, bool FRAG>
__global__ __launch_bounds__(NT) void k_act_scale_quantize(const uint16_t *__restrict__ A, int64_t lda, int M, int K,
                                                           int rw, uint16_t *__restrict__ s_out,
                                                           uint32_t *__restrict__ frag, int s_pad,
                                                           uint32_t *__restrict__ mask, uint32_t *__restrict__ sign,
                                                           int whole)
{
    __shared__ long long s_ll[NT / 64];
    const int m = blockIdx.x, c8 = (K + 7) / 8;
    uint4 x[NG];
    if (m < M) {
        load_row_groups<NG, NT>(A + (int64_t)m * lda, K, c8, whole != 0, x);
    } else {
#pragma unroll
        for (int g = 0; g < NG; ++g) x[g] = make_uint4(0, 0, 0, 0);
    }
    double part = 0.0;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {  // elements past K were loaded as +0 and add nothing
            const uint16_t h = half_of(x[g], i) & 0x7fff;
            const float f = h < 0x7c00 ? half_bits_to_float(h) : 0.0f;  // NaN / Inf stay out
            part += (double)f;
        }
    }
    const long long S = block_sum<NT>(double_units(part), s_ll);
    const uint16_t s_bits = double_to_half_bits((double)S / ((double)K * 8388608.0));  // 2 S / (K 2^24)
    if (threadIdx.x == 0 && m < M) s_out[m] = s_bits;
    // an all-zero (or all non-finite) row has s = 0, an invalid scale: the row ternarises to zero
    const float sc = half_bits_to_float(s_bits);
    const bool ok = sc > 0.0f && sc < __builtin_inff();
    const TernaryThr thr = ternary_thresholds(s_bits, true);
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        const int c = (int)threadIdx.x + NT * g, q = c >> 2, j = c & 3;
        if (FRAG) {
            const uint32_t D = fragment_dword(x[g], thr, j);
            int step, half;
            word_slot(q, step, half);
            if (step < s_pad)
                frag[(((int64_t)(m >> 5) * s_pad + step) * 64 + half * 32 + (m & 31)) * 4 + j] = D;
        } else {
            uint16_t v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = half_of(x[g], i);
            const TernaryBits tb = ternary_bits_fp16(v, 8, 0.5f * sc, ok);
            const uint32_t mw = quad_word(tb.nz, lane), sw = quad_word(tb.neg, lane);
            if (q < rw && j == 0) {
                mask[(int64_t)m * rw + q] = mw;
                sign[(int64_t)m * rw + q] = sw;
            }
        }
    }
}

// mask plane of a binary (+-1) activation matrix: every element is non-zero; pad bits stay zero
__global__ __launch_bounds__(kThreads) void k_full_mask(uint32_t *__restrict__ mask, int64_t words, int rw, int K)
{
    const int64_t gid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (gid >= words) return;
    const int q = (int)(gid % rw), left = K - 32 * q;
    mask[gid] = left >= 32 ? 0xffffffffu : (left > 0 ? (1u << left) - 1u : 0u);
}

}  // namespace

hipError_t launch_full_mask(uint32_t *mask, int M, int K, hipStream_t st)
{
    const int rw = 4 * ((K + 127) / 128);
    const int64_t words = (int64_t)M * rw;
    if (words == 0) return hipSuccess;
    hipLaunchKernelGGL(k_full_mask, dim3((unsigned)((words + kThreads - 1) / kThreads)), dim3(kThreads), 0, st, mask,
                       words, rw, K);
    return hipGetLastError();
}

hipError_t launch_prepare_weights(const void *W, int64_t ldw, int N, int K, uint32_t *wsign, uint16_t *s_w,
                                  hipStream_t st)
{
    if (N == 0) return hipSuccess;
    const int rw = 4 * ((K + 127) / 128);
    const int whole = (((uintptr_t)W % 16) == 0 && (ldw % 8) == 0 && (K % 8) == 0) ? 1 : 0;
    const int c8 = rw * 4;  // 128-bit groups per row; K <= 32768 -> at most 4096
#define BWTA_PREP(NG_, NT_)                                                                                   \
    if (c8 <= NG_ * NT_) {                                                                                    \
        hipLaunchKernelGGL((k_prepare_weights<NG_, NT_>), dim3(N), dim3(NT_), 0, st, (const uint16_t *)W, ldw, K, rw, \
                           wsign, s_w, whole);                                                                \
        return hipGetLastError();                                                                             \
    }
    BWTA_PREP(1, 256) BWTA_PREP(2, 256) BWTA_PREP(4, 256) BWTA_PREP(8, 256) BWTA_PREP(4, 1024)
#undef BWTA_PREP
    return hipErrorInvalidValue;
}

hipError_t launch_act_scale(const void *A, int64_t lda, int M, int K, uint16_t *s, hipStream_t st)
{
    if (M == 0) return hipSuccess;
    const int whole = (((uintptr_t)A % 16) == 0 && (lda % 8) == 0 && (K % 8) == 0) ? 1 : 0;
    const int c8 = (K + 7) / 8;
#define BWTA_SCALE(NG_, NT_)                                                                                       \
    if (c8 <= NG_ * NT_) {                                                                                         \
        hipLaunchKernelGGL((k_act_scale<NG_, NT_>), dim3(M), dim3(NT_), 0, st, (const uint16_t *)A, lda, K, s, whole); \
        return hipGetLastError();                                                                                  \
    }
    BWTA_SCALE(1, 256) BWTA_SCALE(2, 256) BWTA_SCALE(4, 256) BWTA_SCALE(8, 256) BWTA_SCALE(4, 1024)
#undef BWTA_SCALE
    return hipErrorInvalidValue;
}

// scale + ternarised operand in one pass; frag != nullptr selects fragments, else planes
hipError_t launch_act_scale_quantize(const void *A, int64_t lda, int M, int K, uint16_t *s_out, uint32_t *frag,
                                     uint32_t *mask, uint32_t *sign, hipStream_t st)
{
    if (M == 0) return hipSuccess;
    const int rw = 4 * ((K + 127) / 128);
    const int whole = (((uintptr_t)A % 16) == 0 && (lda % 8) == 0 && (K % 8) == 0) ? 1 : 0;
    const int s_pad = fp4_s_pad(rw);
    const int rows = frag ? 32 * fp4_rb_pad(M) : M;
    const int c8 = frag ? 8 * s_pad : 4 * rw;  // 128-bit groups a row's threads must cover (padding included)
#define BWTA_SQ(NG_, NT_)                                                                                          \
    if (c8 <= NG_ * NT_) {                                                                                         \
        if (frag)                                                                                                  \
            hipLaunchKernelGGL((k_act_scale_quantize<NG_, NT_, true>), dim3(rows), dim3(NT_), 0, st,                \
                               (const uint16_t *)A, lda, M, K, rw, s_out, frag, s_pad, mask, sign, whole);         \
        else                                                                                                       \
            hipLaunchKernelGGL((k_act_scale_quantize<NG_, NT_, false>), dim3(rows), dim3(NT_), 0, st,               \
                               (const uint16_t *)A, lda, M, K, rw, s_out, frag, s_pad, mask, sign, whole);         \
        return hipGetLastError();                                                                                  \
    }
    BWTA_SQ(1, 256) BWTA_SQ(2, 256) BWTA_SQ(4, 256) BWTA_SQ(8, 256) BWTA_SQ(4, 1024)
#undef BWTA_SQ
    return hipErrorInvalidValue;
}

hipError_t launch_quantize_pack(const void *A, int dtype, int64_t lda, ScaleArg s_a, int M, int K,
                                uint32_t *mask, uint32_t *sign, int32_t *nnz, hipStream_t st)
{
    const int rw = 4 * ((K + 127) / 128);
    const int64_t total = (int64_t)M * rw * 4;
    if (total == 0) return hipSuccess;
    const unsigned grid = (unsigned)((total + kThreads - 1) / kThreads);
    const int elt = dtype == 0 ? 2 : 1;
    const int vec_ok = (((uintptr_t)A % (8 * elt)) == 0 && (lda % 8) == 0) ? 1 : 0;
    if (dtype == 0 && vec_ok && (K % 8) == 0 && (int64_t)M * rw >= kQuadGroupMinThreads)
        hipLaunchKernelGGL(k_quantize_pack_vec<0>, dim3((unsigned)(((int64_t)M * rw + kThreads - 1) / kThreads)),
                           dim3(kThreads), 0, st, (const uint16_t *)A, lda, s_a, M, K, rw, mask, sign);
    else if (dtype == 0)
        hipLaunchKernelGGL(k_quantize_pack<0>, dim3(grid), dim3(kThreads), 0, st, A, lda, s_a, M, K, rw,
                           mask, sign, vec_ok);
    else
        hipLaunchKernelGGL(k_quantize_pack<1>, dim3(grid), dim3(kThreads), 0, st, A, lda, s_a, M, K, rw,
                           mask, sign, vec_ok);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || nnz == nullptr) return e;
    hipLaunchKernelGGL(k_row_popcount, dim3((M + 3) / 4), dim3(kThreads), 0, st, mask, M, rw, nnz);
    return hipGetLastError();
}

hipError_t launch_quantize_pack_bool(const void *A, int64_t lda, ScaleArg s_a, int M, int K, uint32_t *mask,
                                     hipStream_t st)
{
    const int rw = 4 * ((K + 127) / 128);
    const int64_t total = (int64_t)M * rw * 4;
    if (total == 0) return hipSuccess;
    const unsigned grid = (unsigned)((total + kThreads - 1) / kThreads);
    const int vec_ok = (((uintptr_t)A % 16) == 0 && (lda % 8) == 0) ? 1 : 0;
    if (vec_ok && (K % 8) == 0 && (int64_t)M * rw >= kQuadGroupMinThreads)
        hipLaunchKernelGGL(k_quantize_pack_vec<2>, dim3((unsigned)(((int64_t)M * rw + kThreads - 1) / kThreads)),
                           dim3(kThreads), 0, st, (const uint16_t *)A, lda, s_a, M, K, rw, mask, (uint32_t *)nullptr);
    else
        hipLaunchKernelGGL(k_quantize_pack<2>, dim3(grid), dim3(kThreads), 0, st, A, lda, s_a, M, K, rw, mask,
                           (uint32_t *)nullptr, vec_ok);
    return hipGetLastError();
}

hipError_t launch_pack_weights(const void *W, int dtype, int64_t ldw, int N, int K, uint32_t *wsign,
                               hipStream_t st)
{
    const int rw = 4 * ((K + 127) / 128);
    const int64_t total = (int64_t)N * rw * 4;
    if (total == 0) return hipSuccess;
    const unsigned grid = (unsigned)((total + kThreads - 1) / kThreads);
    const int elt = dtype == 0 ? 2 : 1;
    const int vec_ok = (((uintptr_t)W % (8 * elt)) == 0 && (ldw % 8) == 0) ? 1 : 0;
    if (dtype == 0)
        hipLaunchKernelGGL(k_pack_weights<0>, dim3(grid), dim3(kThreads), 0, st, W, ldw, N, K, rw, wsign,
                           vec_ok);
    else
        hipLaunchKernelGGL(k_pack_weights<1>, dim3(grid), dim3(kThreads), 0, st, W, ldw, N, K, rw, wsign,
                           vec_ok);
    return hipGetLastError();
}

}  // namespace bwta
