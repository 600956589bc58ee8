// The two attention products of the paper's "Basic Layers for Linear and MatMul" section on packed
// operands, batched over heads:
//   BWTA_QK  (Case 3, ternary x ternary):  acc = sum_k q[m,k] k[n,k]
//   BWTA_Att (Case 2, bool x ternary):     acc = sum_k att[m,k] v[n,k]      (att in {0,1})
// Both are  acc = popc(u) - 2 popc(u & (sA ^ sB))  with u = maskA & maskB: a product is non-zero
// where both operands are, and negative where their signs differ.  A boolean operand is a ternary
// one whose sign plane is absent (all zero), which turns the expression into the paper's
// popc(Att & V+) - popc(Att & V-).  Vector ALU, LDS-tiled, wave64: per 32 multiply-accumulates one
// AND, one three-input boolean op and two popcount-accumulates.
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

}  // namespace

hipError_t launch_matmul_tt(const MatmulTTArgs &g, hipStream_t st)
{
    if (g.M == 0 || g.N == 0 || g.batch == 0) return hipSuccess;
    dim3 grid((g.N + BN - 1) / BN, (g.M + BM - 1) / BM, g.batch);
    hipLaunchKernelGGL(k_matmul_tt, grid, dim3(256), 0, st, g);
    return hipGetLastError();
}

}  // namespace bwta
