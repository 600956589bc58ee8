// BWTA product on the vector ALU: acc = popc(mask) - 2 * popc(mask & (sign ^ wsign))
// (Case 1 of the paper's arithmetic rules in its xor form), LDS-tiled, wave64.
// Per 32 multiply-accumulates the inner loop spends one three-input boolean op and one
// popcount-accumulate.
#include "bwta_internal.h"

namespace bwta {

namespace {

constexpr int BM = 64, BN = 64;  // output tile per 256-thread workgroup
constexpr int KT = 16;           // k-words (512 bits) staged per step
constexpr int LDP = KT + 4;      // padded LDS row pitch: 16-byte reads of 16 rows hit 16 bank groups

__global__ __launch_bounds__(256) void k_gemm_popc_tiled(GemmArgs g)
{
    __shared__ __attribute__((aligned(16))) uint32_t sM[BM][LDP];
    __shared__ __attribute__((aligned(16))) uint32_t sS[BM][LDP];
    __shared__ __attribute__((aligned(16))) uint32_t sW[BN][LDP];
    __shared__ int sNnz[BM];

    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int rw = g.rw;

    // nnz of the tile's rows: 4 threads per row stride over the row's words.
    {
        const int r = tid >> 2, part = tid & 3;
        int c = 0;
        if (m0 + r < g.M) {
            const uint32_t *row = g.mask + (int64_t)(m0 + r) * rw;
            for (int w = part; w < rw; w += 4) c += __popc(row[w]);
        }
        c += __shfl_xor(c, 1);
        c += __shfl_xor(c, 2);
        if (part == 0) sNnz[r] = c;
    }

    int cnt[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) cnt[i][j] = 0;

    const int lr = tid >> 2, lq = tid & 3;  // loader: row, 16-byte column
    for (int k0 = 0; k0 < rw; k0 += KT) {
        uint4 vm = make_uint4(0, 0, 0, 0), vs = vm, vw = vm;
        const int kw = k0 + 4 * lq;
        if (kw < rw) {
            if (m0 + lr < g.M) {
                vm = *(const uint4 *)(g.mask + (int64_t)(m0 + lr) * rw + kw);
                vs = *(const uint4 *)(g.sign + (int64_t)(m0 + lr) * rw + kw);
            }
            if (n0 + lr < g.N) vw = *(const uint4 *)(g.wsign + (int64_t)(n0 + lr) * rw + kw);
        }
        __syncthreads();  // previous step's readers are done
        *(uint4 *)&sM[lr][4 * lq] = vm;
        *(uint4 *)&sS[lr][4 * lq] = vs;
        *(uint4 *)&sW[lr][4 * lq] = vw;
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < KT; kk += 4) {
            uint4 am[4], as[4], bw[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                am[i] = *(const uint4 *)&sM[ty + 16 * i][kk];
                as[i] = *(const uint4 *)&sS[ty + 16 * i][kk];
                bw[i] = *(const uint4 *)&sW[tx + 16 * i][kk];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    cnt[i][j] += __popc(am[i].x & (as[i].x ^ bw[j].x));
                    cnt[i][j] += __popc(am[i].y & (as[i].y ^ bw[j].y));
                    cnt[i][j] += __popc(am[i].z & (as[i].z ^ bw[j].z));
                    cnt[i][j] += __popc(am[i].w & (as[i].w ^ bw[j].w));
                }
        }
    }

#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty + 16 * i;
        if (m >= g.M) continue;
        const int nnz = sNnz[ty + 16 * i];
        const float sa = load_scale(g.s_a, m);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx + 16 * j;
            if (n >= g.N) continue;
            const int a = nnz - 2 * cnt[i][j];
            if (g.acc) g.acc[(int64_t)m * g.N + n] = a;
            if (g.out) g.out[(int64_t)m * g.ldo + n] = scaled_to_half(a, sa * load_scale(g.s_w, n));
        }
    }
}

}  // namespace

hipError_t launch_gemm_popc(const GemmArgs &g, hipStream_t st)
{
    if (g.M == 0 || g.N == 0) return hipSuccess;
    dim3 grid((g.N + BN - 1) / BN, (g.M + BM - 1) / BM);
    hipLaunchKernelGGL(k_gemm_popc_tiled, grid, dim3(256), 0, st, g);
    return hipGetLastError();
}

}  // namespace bwta
