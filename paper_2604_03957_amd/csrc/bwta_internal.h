// Internal declarations shared by the HIP translation units of libbwta.so.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bwta {

struct ScaleArg {
    const uint16_t *ptr;  // fp16 bits, device
    int mode;             // BWTA_SCALE_*
};

struct GemmArgs {
    const uint32_t *mask, *sign, *wsign;
    int M, N, K;
    int rw;  // words per packed row
    ScaleArg s_a, s_w;
    int32_t *acc;   // nullable
    uint16_t *out;  // nullable, fp16 bits
    int64_t ldo;
};

// batched ternary x ternary / bool x ternary product (attention MatMuls)
struct MatmulTTArgs {
    const uint32_t *maskA, *signA, *maskB, *signB;  // sign planes nullable (boolean operand)
    int64_t strideA, strideB;                       // words between batches
    int batch, M, N, K, rw;
    ScaleArg s_a, s_b;  // VECTOR: [batch][M] / [batch][N]
    float alpha;
    int32_t *acc;   // nullable, [batch][M][N] with stride_acc
    uint16_t *out;  // nullable, fp16 bits
    int64_t ldo, stride_acc, stride_out;
};

// launchers (each returns the launch's hipError_t)
// popcount_kernel: the vector-ALU comparison kernel instead of the matrix cores
hipError_t launch_matmul_tt(const MatmulTTArgs &g, bool popcount_kernel, hipStream_t st);
hipError_t launch_prepare_weights(const void *W, int64_t ldw, int N, int K, uint32_t *wsign, uint16_t *s_w,
                                  hipStream_t st);
hipError_t launch_full_mask(uint32_t *mask, int M, int K, hipStream_t st);
hipError_t launch_act_scale(const void *A, int64_t lda, int M, int K, uint16_t *s, hipStream_t st);
hipError_t launch_quantize_pack_bool(const void *A, int64_t lda, ScaleArg s_a, int M, int K, uint32_t *mask,
                                     hipStream_t st);
hipError_t launch_quantize_pack(const void *A, int dtype, int64_t lda, ScaleArg s_a, int M, int K,
                                uint32_t *mask, uint32_t *sign, int32_t *nnz, hipStream_t st);
hipError_t launch_pack_weights(const void *W, int dtype, int64_t ldw, int N, int K, uint32_t *wsign,
                               hipStream_t st);
hipError_t launch_gemm_popc(const GemmArgs &g, hipStream_t st);
bool gemv_popc_supported(const GemmArgs &g);
hipError_t launch_gemv_popc(const GemmArgs &g, hipStream_t st);
hipError_t launch_gemv_popc_grouped(const GemmArgs *gs, int count, hipStream_t st);
bool gemv_fp4_supported(const GemmArgs &g);
hipError_t launch_gemv_fp4(const GemmArgs &g, hipStream_t st);
hipError_t launch_gemv_fp4_grouped(const GemmArgs *gs, int count, hipStream_t st);
void set_gemv_fp4_tile(int rpw, int t, int pf);
bool gemm_mfma_supported(const GemmArgs &g);
hipError_t launch_gemm_mfma(const GemmArgs &g, hipStream_t st);

size_t gemm_fp4_frag_bytes(int M, int K);
void set_fp4_tile(int t);
// the whole linear in one launch (short K, fp16 in, fp16 out)
bool linear_fused_supported(const void *A, int64_t lda, const GemmArgs &g);
hipError_t launch_linear_fused(const void *A, int64_t lda, const GemmArgs &g, hipStream_t st);
void set_linear_fused(int mode, int r);
hipError_t launch_att_v_fp4(const GemmArgs &g, const uint32_t *frag, int batch, int64_t w_stride_words,
                            int64_t out_stride, float alpha, hipStream_t st);
void set_gemv_tile(int g, int nch);
hipError_t launch_gemm_fp4(const GemmArgs &g, uint32_t *frag, bool frag_ready, hipStream_t st);
bool gemm_fp4_lds_supported(const GemmArgs &g);
hipError_t launch_gemm_fp4_lds(const GemmArgs &g, const uint32_t *frag, int variant, hipStream_t st);
hipError_t launch_quantize_to_fp4(const void *A, int64_t lda, ScaleArg s_a, int M, int K, uint32_t *frag,
                                  hipStream_t st);
hipError_t launch_act_scale_quantize(const void *A, int64_t lda, int M, int K, uint16_t *s_out, uint32_t *frag,
                                     uint32_t *mask, uint32_t *sign, hipStream_t st);

// Fragment buffer geometry of the FP4 tiled kernel: [row block of 32][k step of 64][lane][4 dwords],
// padded with zeros to a multiple of 8 row blocks and 8 k steps.
inline int fp4_rb_pad(int M) { return ((M + 31) / 32 + 7) / 8 * 8; }
inline int fp4_s_pad(int rw) { return (rw / 2 + 7) / 8 * 8; }

// ---- device helpers -------------------------------------------------------------------------

__device__ __forceinline__ float half_bits_to_float(uint16_t h)
{
    _Float16 f;
    __builtin_memcpy(&f, &h, 2);
    return (float)f;
}

// Which k step and lane half consume plane word q (identical rule in the converter and the GEMM):
// words are taken in groups of 8 (one 256-k chunk); word j of a group feeds step 2*(j/4) + j%2
// of the chunk on lane half (j%4)/2.
__device__ __forceinline__ void word_slot(int q, int &step, int &half)
{
    const int c = q >> 3, j = q & 7;
    step = 4 * c + 2 * (j >> 2) + (j & 1);
    half = (j & 3) >> 1;
}

// ---- ternarisation of binary16 values in packed half precision ---------------------------------
//
// For binary16 x and T > 0 the sums x - pred(T) and -x - T (pred = next value below) are rounded
// once, and a rounded difference of two binary16 values has the sign of the exact one and is zero
// only when they are equal (gradual underflow).  With the result clamped to [0, 1] (NaN clamps to
// 0):   clamp(x - pred(T)) != 0  <=>  x >= T,      clamp(-x - T) != 0  <=>  x < -T,
// which is the paper's threshold rule with T = s / 2, ties and all, at one instruction per two
// elements and side.  T = s / 2 is a binary16 value unless s lies below 2^-13 with an odd last
// bit; such rows compare 2 x (exact, or +-Inf on the correct side) against s instead.
struct TernaryThr {
    uint32_t cp, cn;  // -pred(T) and -T, each in both halves
    bool twice;       // compare 2 x against T = s
};

__device__ __forceinline__ TernaryThr ternary_thresholds(uint32_t s_bits, bool row_valid)
{
    const bool ok = row_valid && s_bits > 0 && s_bits < 0x7c00;  // finite and > 0; anything else: all zero
    const bool halves = s_bits >= 0x0800 || (s_bits & 1) == 0;
    const uint32_t T = s_bits >= 0x0800 ? s_bits - 0x0400 : (halves ? s_bits >> 1 : s_bits);
    const uint32_t Tp = T - 1;
    uint32_t cp = Tp ? (0x8000u | Tp) : 0u;  // +0, not -0, for pred(T) = 0: (-0) + (+0) is +0
    uint32_t cn = 0x8000u | T;
    if (!ok) cp = cn = 0xfc00u;  // -Inf: every sum is -Inf or NaN
    TernaryThr t;
    t.cp = cp * 0x10001u;
    t.cn = cn * 0x10001u;
    t.twice = ok && !halves;
    return t;
}

// 8 fp16 values of one row (lane j of a quad holds elements 8 j .. 8 j + 7 of a 32-element word) ->
// the dword this lane contributes to the word's fragment: nibble i of dword d holds element
// 4 i + d (bit 1 = non-zero, bit 3 = negative).
__device__ __forceinline__ uint32_t fragment_dword(const uint4 &x, const TernaryThr &t, int j)
{
    uint32_t w[4] = {x.x, x.y, x.z, x.w};  // elements (0,1) (2,3) (4,5) (6,7)
    if (t.twice) {
#pragma unroll
        for (int d = 0; d < 4; ++d) asm("v_pk_add_f16 %0, %1, %1" : "=v"(w[d]) : "v"(w[d]));
    }
    uint32_t one2 = 0x00010001u;
    // byte 0 = elements 0 (low nibble) and 4 (high), byte 1 = 2 and 6, byte 2 = 1 and 5, byte 3 = 3 and 7
    uint32_t V = 0;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        uint32_t p, n, gp, gn;
        asm("v_pk_add_f16 %0, %1, %2 clamp" : "=v"(p) : "v"(w[d]), "v"(t.cp));
        asm("v_pk_add_f16 %0, %1, %2 neg_lo:[1,0] neg_hi:[1,0] clamp" : "=v"(n) : "v"(w[d]), "v"(t.cn));
        asm("v_pk_min_u16 %0, %1, %2" : "=v"(gp) : "v"(p), "v"(one2));  // 1 where x >= T
        asm("v_pk_min_u16 %0, %1, %2" : "=v"(gn) : "v"(n), "v"(one2));  // 1 where x < -T
        const uint32_t sel = __umul24(gn, 5u) + gp;  // per half: non-zero bit, and two places up the sign bit
        const int sh = d == 0 ? 1 : d == 1 ? 9 : d == 2 ? 5 : 13;
        V = (sel << sh) | V;
    }
    // quad byte transpose: lane d of the quad collects the byte holding elements d and d + 4 of
    // every lane -> dword d of the word
    const uint32_t x0 = __builtin_amdgcn_mov_dpp(V, 0x00, 0xf, 0xf, true);  // quad_perm [0,0,0,0]
    const uint32_t x1 = __builtin_amdgcn_mov_dpp(V, 0x55, 0xf, 0xf, true);  // [1,1,1,1]
    const uint32_t x2 = __builtin_amdgcn_mov_dpp(V, 0xaa, 0xf, 0xf, true);  // [2,2,2,2]
    const uint32_t x3 = __builtin_amdgcn_mov_dpp(V, 0xff, 0xf, 0xf, true);  // [3,3,3,3]
    const uint32_t b = ((j & 1) << 1) | (j >> 1);                // the byte with elements j and j + 4
    const uint32_t pick = 0x0c0c0000u | ((4u + b) << 8) | b;      // byte b of the second, then of the first source
    const uint32_t lo = __builtin_amdgcn_perm(x1, x0, pick);     // [x0.b, x1.b, 0, 0]
    const uint32_t hi = __builtin_amdgcn_perm(x3, x2, pick);
    return __builtin_amdgcn_perm(hi, lo, 0x05040100u);
}

__device__ __forceinline__ float load_scale(const ScaleArg &s, int row)
{
    if (s.mode == 0 || s.ptr == nullptr) return 1.0f;
    return half_bits_to_float(s.ptr[s.mode == 1 ? 0 : row]);
}

// fp16( a * s ) with a single rounding.  a is an exact integer-valued float (|a| < 2^24) and
// s = s_a * s_w is exact in fp32 (two 11-bit significands).  v_fma_mixlo_f16 / v_fma_mixhi_f16
// evaluate the fused multiply-add exactly and round once, to nearest even, straight to fp16
// (checked on MI355X against products whose fp32 rounding would sit on an fp16 tie).  The addend
// is -0.0 so that a zero product keeps its sign.
__device__ __forceinline__ uint32_t scaled_to_half2(float a0, float s0, float a1, float s1)
{
    uint32_t r;
    const float nz = -0.0f;
    asm("v_fma_mixlo_f16 %0, %1, %2, %3" : "=v"(r) : "v"(a0), "v"(s0), "v"(nz));
    asm("v_fma_mixhi_f16 %0, %1, %2, %3" : "+v"(r) : "v"(a1), "v"(s1), "v"(nz));
    return r;  // low half = fp16(a0 * s0), high half = fp16(a1 * s1)
}

__device__ __forceinline__ uint16_t scaled_to_half(float a, float s)
{
    uint32_t r;
    const float nz = -0.0f;
    asm("v_fma_mixlo_f16 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(s), "v"(nz));
    return (uint16_t)(r & 0xffffu);
}

__device__ __forceinline__ uint16_t scaled_to_half(int acc, float s) { return scaled_to_half((float)acc, s); }

// Epilogue shared by the matrix-core kernels.  A wavefront owns WM x WN blocks of 32 x 32
// accumulators in the MFMA layout (lane = column r32 of a block, register v = row
// 8*(v/4) + 4*h + v%4).  Scaled fp16 results go through a wavefront-private LDS strip of 32 rows
// so that global stores are 16 bytes per lane along rows; int32 accumulators (optional output,
// used by tests) are stored directly.
//   get(i, j, v)  -> exact int32 accumulator
//   strip         -> this wavefront's LDS scratch, 32 * (32*WN + 8) halfs
//   sa_lds        -> float s_a of the block's rows (index = row within block), filled by caller
template <int WM, int WN, typename Get>
__device__ __forceinline__ void store_wave_tile(const GemmArgs &g, int m_wave, int n_wave, int row_in_block0,
                                                uint16_t *strip, const float *sa_lds, Get get)
{
    constexpr int PITCH = 32 * WN + 8;  // halfs
    const int lane = threadIdx.x & 63, r32 = lane & 31, h = lane >> 5;
    if (g.acc) {
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            const int n = n_wave + 32 * j + r32;
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = m_wave + 32 * i + 8 * (v >> 2) + 4 * h + (v & 3);
                    if (m < g.M && n < g.N) g.acc[(int64_t)m * g.N + n] = get(i, j, v);
                }
        }
    }
    if (!g.out) return;
    float sw[WN];
#pragma unroll
    for (int j = 0; j < WN; ++j) {
        const int n = n_wave + 32 * j + r32;
        sw[j] = n < g.N ? load_scale(g.s_w, n) : 0.0f;
    }
    const bool vec_ok = ((g.ldo & 7) == 0) && (((uintptr_t)g.out & 15) == 0);
    constexpr int LPR = 4 * WN;        // lanes per row when each lane moves 8 halfs
    constexpr int RPI = 64 / LPR;      // rows per store instruction
#pragma unroll
    for (int i = 0; i < WM; ++i) {
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = 8 * (v >> 2) + 4 * h + (v & 3);
                const float sa = sa_lds[row_in_block0 + 32 * i + row];
                strip[row * PITCH + 32 * j + r32] = scaled_to_half(get(i, j, v), sa * sw[j]);
            }
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
        for (int rr = 0; rr < 32; rr += RPI) {
            const int row = rr + lane / LPR, c8 = 8 * (lane % LPR);
            const int m = m_wave + 32 * i + row, n = n_wave + c8;
            if (m < g.M && n < g.N) {
                const uint4 q = *(const uint4 *)(strip + row * PITCH + c8);
                uint16_t *dst = g.out + (int64_t)m * g.ldo + n;
                if (vec_ok && n + 8 <= g.N) {
                    *(uint4 *)dst = q;
                } else {
                    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (n + e < g.N) dst[e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    }
}

}  // namespace bwta
