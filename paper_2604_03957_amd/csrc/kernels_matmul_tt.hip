// The two attention products of the paper's "Basic Layers for Linear and MatMul" section on packed
// operands, batched over heads:
//   BWTA_QK  (Case 3, ternary x ternary):  acc = sum_k q[m,k] k[n,k]
//   BWTA_Att (Case 2, bool x ternary):     acc = sum_k att[m,k] v[n,k]      (att in {0,1})
// Both are  acc = popc(u) - 2 popc(u & (sA ^ sB))  with u = maskA & maskB: a product is non-zero
// where both operands are, and negative where their signs differ.  A boolean operand is a ternary
// one whose sign plane is absent (all zero), which turns the expression into the paper's
// popc(Att & V+) - popc(Att & V-).
//
// Two kernels compute it.  k_matmul_tt_fp4 (the default) runs the product on the FP4 matrix cores:
// +1, -1 and 0 are exact E2M1 values and every partial sum is an integer below 2^24, so the fp32
// accumulators of v_mfma_f32_32x32x64_f8f6f4 hold the popcount result exactly.  Both operands stay
// bit planes in HBM and LDS and are expanded to nibbles in registers.  k_matmul_tt is the vector-ALU
// form (LDS-tiled, wave64: per 32 multiply-accumulates one AND, one three-input boolean op and two
// popcount-accumulates), kept as the comparison path.
#include <type_traits>

#include "bwta_internal.h"

namespace bwta {

namespace {

constexpr int BM = 64, BN = 64;  // output tile per 256-thread workgroup
constexpr int KT = 16;           // k-words (512 bits) staged per step
constexpr int LDP = KT + 4;      // padded LDS row pitch

__global__ __launch_bounds__(256) void k_matmul_tt(MatmulTTArgs g)
{
    __shared__ __attribute__((aligned(16))) uint32_t sAm[BM][LDP];
    __shared__ __attribute__((aligned(16))) uint32_t sAs[BM][LDP];
    __shared__ __attribute__((aligned(16))) uint32_t sBm[BN][LDP];
    __shared__ __attribute__((aligned(16))) uint32_t sBs[BN][LDP];

    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN, b = blockIdx.z;
    const int rw = g.rw;
    const uint32_t *maskA = g.maskA + (int64_t)b * g.strideA, *signA = g.signA ? g.signA + (int64_t)b * g.strideA : nullptr;
    const uint32_t *maskB = g.maskB + (int64_t)b * g.strideB, *signB = g.signB ? g.signB + (int64_t)b * g.strideB : nullptr;

    int both[4][4], diff[4][4];  // popc(u), popc(u & (sA ^ sB))
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) both[i][j] = diff[i][j] = 0;

    const int lr = tid >> 2, lq = tid & 3;  // loader: row, 16-byte column
    for (int k0 = 0; k0 < rw; k0 += KT) {
        const uint4 z = make_uint4(0, 0, 0, 0);
        uint4 am = z, as = z, bm = z, bs = z;
        const int kw = k0 + 4 * lq;
        if (kw < rw) {
            if (m0 + lr < g.M) {
                am = *(const uint4 *)(maskA + (int64_t)(m0 + lr) * rw + kw);
                if (signA) as = *(const uint4 *)(signA + (int64_t)(m0 + lr) * rw + kw);
            }
            if (n0 + lr < g.N) {
                bm = *(const uint4 *)(maskB + (int64_t)(n0 + lr) * rw + kw);
                if (signB) bs = *(const uint4 *)(signB + (int64_t)(n0 + lr) * rw + kw);
            }
        }
        __syncthreads();  // previous step's readers are done
        *(uint4 *)&sAm[lr][4 * lq] = am;
        *(uint4 *)&sAs[lr][4 * lq] = as;
        *(uint4 *)&sBm[lr][4 * lq] = bm;
        *(uint4 *)&sBs[lr][4 * lq] = bs;
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < KT; kk += 4) {
            if (k0 + kk >= rw) break;  // short rows (head dimension 128 = 4 words): skip the zero padding
            uint4 xam[4], xas[4], xbm[4], xbs[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                xam[i] = *(const uint4 *)&sAm[ty + 16 * i][kk];
                xas[i] = *(const uint4 *)&sAs[ty + 16 * i][kk];
                xbm[i] = *(const uint4 *)&sBm[tx + 16 * i][kk];
                xbs[i] = *(const uint4 *)&sBs[tx + 16 * i][kk];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    uint32_t u;
                    u = xam[i].x & xbm[j].x; both[i][j] += __popc(u); diff[i][j] += __popc(u & (xas[i].x ^ xbs[j].x));
                    u = xam[i].y & xbm[j].y; both[i][j] += __popc(u); diff[i][j] += __popc(u & (xas[i].y ^ xbs[j].y));
                    u = xam[i].z & xbm[j].z; both[i][j] += __popc(u); diff[i][j] += __popc(u & (xas[i].z ^ xbs[j].z));
                    u = xam[i].w & xbm[j].w; both[i][j] += __popc(u); diff[i][j] += __popc(u & (xas[i].w ^ xbs[j].w));
                }
        }
    }

    // out = fp16( acc * s ),  s = fp32( alpha * (s_a * s_b) ): s_a * s_b is exact in fp32, the
    // multiplication by alpha rounds once, and acc * s is rounded once more, to fp16
    int32_t *acc = g.acc ? g.acc + (int64_t)b * g.stride_acc : nullptr;
    uint16_t *out = g.out ? g.out + (int64_t)b * g.stride_out : nullptr;
    const ScaleArg sa{g.s_a.ptr && g.s_a.mode == 2 ? g.s_a.ptr + (int64_t)b * g.M : g.s_a.ptr, g.s_a.mode};
    const ScaleArg sb{g.s_b.ptr && g.s_b.mode == 2 ? g.s_b.ptr + (int64_t)b * g.N : g.s_b.ptr, g.s_b.mode};
    // int32 results (tests, debugging) go out directly; fp16 results are gathered in LDS so that the
    // tile leaves as 16-byte row-contiguous stores (the score matrix is the bulk of the traffic)
    __shared__ __attribute__((aligned(16))) uint16_t sOut[BM][BN + 8];
    const bool vec_ok = out && ((g.ldo & 7) == 0) && ((g.stride_out & 7) == 0) && (((uintptr_t)g.out & 15) == 0) &&
                        (n0 + BN <= g.N);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty + 16 * i;
        const float fa = m < g.M ? load_scale(sa, m) : 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx + 16 * j;
            const int a = both[i][j] - 2 * diff[i][j];
            if (m < g.M && n < g.N) {
                if (acc) acc[(int64_t)m * g.N + n] = a;
                if (out) {
                    const uint16_t h = scaled_to_half(a, g.alpha * (fa * load_scale(sb, n)));
                    if (vec_ok)
                        sOut[ty + 16 * i][tx + 16 * j] = h;
                    else
                        out[(int64_t)m * g.ldo + n] = h;
                }
            }
        }
    }
    if (vec_ok) {  // uniform over the workgroup
        __syncthreads();
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int p = tid + 256 * r, row = p >> 3, c8 = 8 * (p & 7);  // 64 rows x 8 pieces of 8 halfs
            if (m0 + row < g.M)
                *(uint4 *)(out + (int64_t)(m0 + row) * g.ldo + n0 + c8) = *(const uint4 *)&sOut[row][c8];
        }
    }
}


// ---- matrix-core form -------------------------------------------------------------------------
// Workgroup = 4 wavefronts (2 x 2) on a 128 x 128 output tile, a wavefront owns 2 x 2 blocks of
// 32 x 32.  K advances in slabs of 256 (8 plane words per row); a slab of the four planes sits in
// LDS (double-buffered, one barrier per slab).  Lane (r32, h) of an operand block holds row r32
// and, for step s of the slab, plane word 4 h + s: a dot product is unchanged by a permutation of
// k applied to both operands, so a lane may take four consecutive words (one 16-byte LDS read per
// plane) and deal bit 4 n + d of a word to nibble n of dword d.  The B rows are the instruction's
// first operand, so a lane ends with four consecutive n of one m and the tile leaves as 16-byte
// row-contiguous stores.
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));

constexpr int FT = 128;                 // tile edge
constexpr int FSW = 8;                  // plane words per slab
constexpr int FPITCH = 12;              // dwords per LDS row: 16-byte reads at stride 48 B are conflict-free
constexpr int FPLANE = FT * FPITCH;     // dwords per plane tile
constexpr int FSTAGE = 4 * FPLANE;      // Am, As, Bm, Bs
constexpr int FSTRIP_PITCH = 64 + 8;    // halfs per row of a wavefront's output strip
constexpr int FSMEM_BYTES = 2 * FSTAGE * 4 + 2 * FT * 4;  // two stages, then [128] s_b and [128] s_a as floats

// plane words -> E2M1 nibbles (+1 = 0b0010, -1 = 0b1010, 0 = 0b0000): bit 4 n + d -> nibble n of dword d
template <bool SIGNED>
__device__ __forceinline__ v8i widen_t(uint32_t m, uint32_t s, uint32_t m88, uint32_t c22)
{
    v8i r;
    if (SIGNED) {
        const uint32_t ss = s & m;
        r[0] = (int)(((ss << 3) & m88) | ((m << 1) & c22));
        r[1] = (int)(((ss << 2) & m88) | (m & c22));
        r[2] = (int)(((ss << 1) & m88) | ((m >> 1) & c22));
        r[3] = (int)((ss & m88) | ((m >> 2) & c22));
    } else {
        r[0] = (int)((m << 1) & c22);
        r[1] = (int)(m & c22);
        r[2] = (int)((m >> 1) & c22);
        r[3] = (int)((m >> 2) & c22);
    }
    r[4] = r[5] = r[6] = r[7] = 0;
    return r;
}

template <bool SIGN_A, bool SIGN_B>
__global__ __launch_bounds__(256, 2) void k_matmul_tt_fp4(MatmulTTArgs g)
{
    extern __shared__ __attribute__((aligned(16))) uint32_t fsm[];
    float *sc_lds = (float *)(fsm + 2 * FSTAGE);  // [FT] s_b, then [FT] s_a
    const int tid = threadIdx.x, lane = tid & 63, wl = tid >> 6;
    const int wm = wl >> 1, wn = wl & 1, r32 = lane & 31, h = lane >> 5;
    const int m0 = blockIdx.y * FT, n0 = blockIdx.x * FT, b = blockIdx.z;
    const int rw = g.rw;
    const uint32_t *planes[4] = {g.maskA + (int64_t)b * g.strideA, SIGN_A ? g.signA + (int64_t)b * g.strideA : nullptr,
                                 g.maskB + (int64_t)b * g.strideB, SIGN_B ? g.signB + (int64_t)b * g.strideB : nullptr};

    // scales: requested first by every thread (without a scale: a dropped read), parked in LDS with
    // the first slab, so neither the operand requests nor the epilogue wait for them
    const ScaleArg sa{g.s_a.ptr && g.s_a.mode == 2 ? g.s_a.ptr + (int64_t)b * g.M : g.s_a.ptr, g.s_a.ptr ? g.s_a.mode : 0};
    const ScaleArg sb{g.s_b.ptr && g.s_b.mode == 2 ? g.s_b.ptr + (int64_t)b * g.N : g.s_b.ptr, g.s_b.ptr ? g.s_b.mode : 0};
    const int sidx = tid & (FT - 1);
    const bool is_b = tid < FT;
    const ScaleArg &mine = is_b ? sb : sa;
    const bool want = is_b ? n0 + sidx < g.N : m0 + sidx < g.M;
    const bool have = want && mine.mode != 0;
    const uint16_t sc_bits = *(have ? mine.ptr + (mine.mode == 1 ? 0 : (is_b ? n0 : m0) + sidx) : (const uint16_t *)g.maskA);
    __builtin_amdgcn_sched_barrier(0);

    // slab loader: plane pl, 128 rows x 2 pieces of 16 bytes; thread t takes piece t of every plane
    const int lrow = tid >> 1, lcol = tid & 1;
    auto fetch = [&](int slab, uint4(&dst)[4]) {
        const int kw = slab * FSW + 4 * lcol;
#pragma unroll
        for (int pl = 0; pl < 4; ++pl) {
            dst[pl] = make_uint4(0, 0, 0, 0);
            if ((pl == 1 && !SIGN_A) || (pl == 3 && !SIGN_B)) continue;
            const int row = (pl < 2 ? m0 : n0) + lrow, rows = pl < 2 ? g.M : g.N;
            // rows and words outside the operand re-read its first bytes and are zeroed when staged
            const bool inside = row < rows && kw < rw;
            dst[pl] = *(const uint4 *)(planes[pl] + (inside ? (int64_t)row * rw + kw : 0));
        }
    };
    auto stage = [&](int buf, int slab, const uint4(&src)[4]) {
        const int kw = slab * FSW + 4 * lcol;
#pragma unroll
        for (int pl = 0; pl < 4; ++pl) {
            if ((pl == 1 && !SIGN_A) || (pl == 3 && !SIGN_B)) continue;
            const int row = (pl < 2 ? m0 : n0) + lrow, rows = pl < 2 ? g.M : g.N;
            const bool inside = row < rows && kw < rw;
            *(uint4 *)(fsm + buf * FSTAGE + pl * FPLANE + lrow * FPITCH + 4 * lcol) = inside ? src[pl] : make_uint4(0, 0, 0, 0);
        }
    };

    uint32_t m88 = 0x88888888u, c22 = 0x22222222u;  // opaque, so each expansion is one v_and_or_b32
    asm volatile("" : "+s"(m88));
    asm volatile("" : "+v"(c22));

    v16f acc[2][2];  // [n block][m block]
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][i][v] = 0.0f;

    const int nslab = (rw + FSW - 1) / FSW;
    // A full slab: lane (r32, h) takes words 4 h .. 4 h + 3 of its row, one per step.  A last slab
    // that holds only four words (K = 128: the whole row) deals them as words 2 h, 2 h + 1 over two
    // steps instead, so no instruction runs on an operand half made of padding.
    auto compute = [&](int buf, auto half_slab) {
        constexpr bool HALF = decltype(half_slab)::value;
        constexpr int NS = HALF ? 2 : 4;
        const uint32_t *st = fsm + buf * FSTAGE;
        uint32_t am[2][NS], as[2][NS], bm[2][NS], bs[2][NS];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int ra = (wm * 64 + 32 * i + r32) * FPITCH + NS * h, rb = (wn * 64 + 32 * i + r32) * FPITCH + NS * h;
            if (HALF) {
                const uint2 a0 = *(const uint2 *)(st + ra), b0 = *(const uint2 *)(st + 2 * FPLANE + rb);
                am[i][0] = a0.x, am[i][1] = a0.y, bm[i][0] = b0.x, bm[i][1] = b0.y;
                if (SIGN_A) {
                    const uint2 a1 = *(const uint2 *)(st + FPLANE + ra);
                    as[i][0] = a1.x, as[i][1] = a1.y;
                }
                if (SIGN_B) {
                    const uint2 b1 = *(const uint2 *)(st + 3 * FPLANE + rb);
                    bs[i][0] = b1.x, bs[i][1] = b1.y;
                }
            } else {
                const v4u a0 = *(const v4u *)(st + ra), b0 = *(const v4u *)(st + 2 * FPLANE + rb);
#pragma unroll
                for (int s = 0; s < NS; ++s) am[i][s] = a0[s], bm[i][s] = b0[s];
                if (SIGN_A) {
                    const v4u a1 = *(const v4u *)(st + FPLANE + ra);
#pragma unroll
                    for (int s = 0; s < NS; ++s) as[i][s] = a1[s];
                }
                if (SIGN_B) {
                    const v4u b1 = *(const v4u *)(st + 3 * FPLANE + rb);
#pragma unroll
                    for (int s = 0; s < NS; ++s) bs[i][s] = b1[s];
                }
            }
        }
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            v8i fa[2], fb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                fa[i] = widen_t<SIGN_A>(am[i][s], SIGN_A ? as[i][s] : 0u, m88, c22);
                fb[i] = widen_t<SIGN_B>(bm[i][s], SIGN_B ? bs[i][s] : 0u, m88, c22);
            }
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    acc[j][i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb[j], fa[i], acc[j][i], 4, 4, 0, 0, 0, 0);
        }
    };
    // One slab is requested ahead (registers) while the current one is multiplied out of LDS; one
    // barrier per slab.  The last iteration re-requests its own slab, so every iteration issues
    // the same loads.  (Requesting two slabs ahead was measured: no faster on Att V, slower on Q K^T.)
    uint4 pre[4];
    fetch(0, pre);
    __builtin_amdgcn_sched_barrier(0);
    stage(0, 0, pre);
    sc_lds[tid] = have ? half_bits_to_float(sc_bits) : (want ? 1.0f : 0.0f);
    __syncthreads();
    int buf = 0;
    const int nfull = rw / FSW;  // rw is a multiple of 4: what is left after the full slabs is one half slab
    for (int it = 0; it < nfull; ++it) {
        const int nxt = it + 1 < nslab ? it + 1 : nslab - 1;
        fetch(nxt, pre);
        compute(buf, std::false_type{});
        stage(buf ^ 1, nxt, pre);
        __syncthreads();
        buf ^= 1;
    }
    if (nfull < nslab) {  // staged by the last iteration (or by the prologue when it is the only slab)
        compute(buf, std::true_type{});
        __syncthreads();  // the epilogue's strips reuse the slab memory
    }

    // ---- epilogue.  Lane (r32, h) of block (j, i) holds m = 32 i + r32 and n = 32 j + 8 q + 4 h + e
    // (register v = 4 q + e).
    const int m_wave = m0 + wm * 64, n_wave = n0 + wn * 64;
    if (g.acc) {
        int32_t *accp = g.acc + (int64_t)b * g.stride_acc;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int m = m_wave + 32 * i + r32;
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int n = n_wave + 32 * j + 8 * (v >> 2) + 4 * h + (v & 3);
                    if (m < g.M && n < g.N) accp[(int64_t)m * g.N + n] = (int)acc[j][i][v];
                }
        }
    }
    if (!g.out) return;
    uint16_t *out = g.out + (int64_t)b * g.stride_out;
    // out = fp16( acc * s ),  s = fp32( alpha * (s_a * s_b) ): s_a * s_b is exact in fp32, the
    // multiplication by alpha rounds once, and acc * s is rounded once more, to fp16.
    // The loop's last barrier retired every read of the slabs, whose LDS the strips reuse.
    uint16_t *strip = (uint16_t *)fsm + wl * (32 * FSTRIP_PITCH);
    const float *sb_lds = sc_lds, *sa_lds = sc_lds + FT;
    const bool full = (m_wave + 64 <= g.M) && (n_wave + 64 <= g.N) && ((g.ldo & 7) == 0) &&
                      (g.batch == 1 || (g.stride_out & 7) == 0) && (((uintptr_t)g.out & 15) == 0);
    // Layerwise (scalar or absent) scales on both sides make the factor one number for the whole
    // launch; per-row scales cost two multiplications per element, which is what bounds Q K^T.
    const bool one_factor = sa.mode != 2 && sb.mode != 2;
    const float factor = g.alpha * (sa_lds[0] * sb_lds[0]);  // row m0 and column n0 exist
    auto write_out = [&](auto uniform) {
        constexpr bool UNI = decltype(uniform)::value;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const float fa = sa_lds[wm * 64 + 32 * i + r32];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int nl = 32 * j + 8 * q + 4 * h;
                    float s0 = factor, s1 = factor, s2 = factor, s3 = factor;
                    if (!UNI) {
                        const float4 fb = *(const float4 *)(sb_lds + wn * 64 + nl);
                        s0 = g.alpha * (fa * fb.x), s1 = g.alpha * (fa * fb.y);
                        s2 = g.alpha * (fa * fb.z), s3 = g.alpha * (fa * fb.w);
                    }
                    uint2 hv;
                    hv.x = scaled_to_half2(acc[j][i][4 * q], s0, acc[j][i][4 * q + 1], s1);
                    hv.y = scaled_to_half2(acc[j][i][4 * q + 2], s2, acc[j][i][4 * q + 3], s3);
                    *(uint2 *)(strip + r32 * FSTRIP_PITCH + nl) = hv;
                }
            }
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
            for (int rr = 0; rr < 32; rr += 8) {
                const int row = rr + (lane >> 3), c8 = 8 * (lane & 7);
                const int mo = m_wave + 32 * i + row, n = n_wave + c8;
                const uint4 qd = *(const uint4 *)(strip + row * FSTRIP_PITCH + c8);
                uint16_t *dst = out + (int64_t)mo * g.ldo + n;
                if (full) {
                    const v4u qv = {qd.x, qd.y, qd.z, qd.w};
                    __builtin_nontemporal_store(qv, (v4u *)dst);  // streamed once, never re-read here
                } else if (mo < g.M && n < g.N) {
                    const uint32_t w[4] = {qd.x, qd.y, qd.z, qd.w};
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (n + e < g.N) dst[e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
                }
            }
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        }
    };
    if (one_factor)
        write_out(std::true_type{});
    else
        write_out(std::false_type{});
}

template <bool SIGN_A, bool SIGN_B>
hipError_t launch_fp4_t(const MatmulTTArgs &g, hipStream_t st)
{
    dim3 grid((g.N + FT - 1) / FT, (g.M + FT - 1) / FT, g.batch);
    hipLaunchKernelGGL((k_matmul_tt_fp4<SIGN_A, SIGN_B>), grid, dim3(256), FSMEM_BYTES, st, g);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_matmul_tt(const MatmulTTArgs &g, bool popcount_kernel, hipStream_t st)
{
    if (g.M == 0 || g.N == 0 || g.batch == 0) return hipSuccess;
    if (!popcount_kernel) {
        if (g.signA && g.signB) return launch_fp4_t<true, true>(g, st);
        if (g.signA) return launch_fp4_t<true, false>(g, st);
        if (g.signB) return launch_fp4_t<false, true>(g, st);
        return launch_fp4_t<false, false>(g, st);
    }
    dim3 grid((g.N + BN - 1) / BN, (g.M + BM - 1) / BM, g.batch);
    hipLaunchKernelGGL(k_matmul_tt, grid, dim3(256), 0, st, g);
    return hipGetLastError();
}

}  // namespace bwta
