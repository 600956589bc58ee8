// BWTA product on the int8 matrix cores (v_mfma_i32_32x32x32_i8), fed from the 1-bit planes.
//
// Operands stay bit-packed all the way into LDS; each lane widens the bits it needs to int8
// with a couple of AND/shift ops per register, using two facts:
//   * a dot product does not care about the order of k, so the bits of a packed word may be
//     dealt to the instruction's k slots in whatever order makes widening cheapest, as long as
//     both operands use the same order;
//   * a byte holding a single bit at position p is the int8 value 2^p.  If the weight bit sits
//     at position b and the activation code at position a with a + b = 5 in every slot, all
//     products carry the same factor 32, which is shifted out exactly at the end.
// The activation enters as u = t + 1 in {0, 1, 2} (a 2-bit code: bit0 = "is zero", bit1 = "is
// +1"), the weight as its sign bit s in {0, 1} (w = 1 - 2 s).  With G = 32 * sum_k u_k s_k the
// matrix cores deliver, the exact BWTA product (Case 1 of the paper's arithmetic rules) is
//     acc = sum_k t_k w_k = T_m + 2 B_n - G / 16,   T_m = sum_k t_k,  B_n = sum_k s_k,
// and T_m, B_n are counted by the threads that stage the tiles.
#include "bwta_internal.h"

namespace bwta {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int KT = 16;        // plane words (512 k) staged per step
constexpr int A_PITCH = 36;   // dwords per LDS row of activation codes: 4 blocks * 8 + 4 pad
constexpr int W_PITCH = 18;   // dwords per LDS row of weight words: 16 + 2 pad

// 2-bit codes of one plane word: ue holds elements at even in-byte positions, uo the odd ones,
// field f (bits 2f, 2f+1 of each byte) <-> in-byte position 2f (+1).
__device__ __forceinline__ void make_codes(uint32_t m, uint32_t s, uint32_t &ue, uint32_t &uo)
{
    const uint32_t z = ~m, p = m & ~s;
    ue = (z & 0x55555555u) | ((p & 0x55555555u) << 1);
    uo = ((z >> 1) & 0x55555555u) | (p & 0xAAAAAAAAu);
}

// activation operand: slot d carries u * 2^a, a = {0, 2, 4, 5}
__device__ __forceinline__ v4i widen_act(uint32_t u)
{
    v4i r;
    r.x = (int)(u & 0x03030303u);
    r.y = (int)(u & 0x0C0C0C0Cu);
    r.z = (int)(u & 0x30303030u);
    r.w = (int)((u >> 1) & 0x60606060u);
    return r;
}

// weight operand: slot d carries s * 2^b, b = {5, 3, 1, 0}; even / odd in-byte positions
__device__ __forceinline__ v4i widen_w_even(uint32_t x)
{
    v4i r;
    r.x = (int)((x << 5) & 0x20202020u);
    r.y = (int)((x << 1) & 0x08080808u);
    r.z = (int)((x >> 3) & 0x02020202u);
    r.w = (int)((x >> 6) & 0x01010101u);
    return r;
}
__device__ __forceinline__ v4i widen_w_odd(uint32_t x)
{
    v4i r;
    r.x = (int)((x << 4) & 0x20202020u);
    r.y = (int)(x & 0x08080808u);
    r.z = (int)((x >> 4) & 0x02020202u);
    r.w = (int)((x >> 7) & 0x01010101u);
    return r;
}

template <int WM, int WN>
struct Tile {
    static constexpr int BM = 64 * WM, BN = 64 * WN;  // 2 x 2 waves, each WM x WN blocks of 32 x 32
    static constexpr int BUF_DWORDS = BM * A_PITCH + BN * W_PITCH;
    static constexpr int SMEM_BYTES = (2 * BUF_DWORDS + BM + BN) * 4;
};

template <int WM, int WN>
__global__ __launch_bounds__(256, 1) void k_gemm_mfma(GemmArgs g)
{
    using T = Tile<WM, WN>;
    extern __shared__ __attribute__((aligned(16))) uint32_t smem[];
    int *sT = (int *)(smem + 2 * T::BUF_DWORDS);
    int *sB = sT + T::BM;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int r32 = lane & 31, h = lane >> 5;
    const int m0 = blockIdx.y * T::BM, n0 = blockIdx.x * T::BN;
    const int rw = g.rw;
    const int lr = tid >> 2, lq = tid & 3;  // loader: row within a group of 64, 128-bit column

    uint4 pm[WM], ps[WM], pw[WN];  // prefetch registers
    int tsum[WM], bsum[WN];
#pragma unroll
    for (int i = 0; i < WM; ++i) tsum[i] = 0;
#pragma unroll
    for (int i = 0; i < WN; ++i) bsum[i] = 0;

    auto fetch = [&](int k0) {
        const int kw = k0 + 4 * lq;
        const bool kin = kw < rw;
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            const int m = m0 + lr + 64 * i;
            pm[i] = make_uint4(0, 0, 0, 0);
            ps[i] = pm[i];
            if (kin && m < g.M) {
                pm[i] = *(const uint4 *)(g.mask + (int64_t)m * rw + kw);
                ps[i] = *(const uint4 *)(g.sign + (int64_t)m * rw + kw);
            }
        }
#pragma unroll
        for (int i = 0; i < WN; ++i) {
            const int n = n0 + lr + 64 * i;
            pw[i] = make_uint4(0, 0, 0, 0);
            if (kin && n < g.N) pw[i] = *(const uint4 *)(g.wsign + (int64_t)n * rw + kw);
        }
    };

    auto stage = [&](int buf) {
        uint32_t *sA = smem + buf * T::BUF_DWORDS;
        uint32_t *sW = sA + T::BM * A_PITCH;
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            const uint32_t mk[4] = {pm[i].x, pm[i].y, pm[i].z, pm[i].w};
            const uint32_t sg[4] = {ps[i].x, ps[i].y, ps[i].z, ps[i].w};
            uint32_t c[8];
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                make_codes(mk[w], sg[w], c[2 * w], c[2 * w + 1]);
                tsum[i] += __popc(mk[w]) - 2 * __popc(mk[w] & sg[w]);
            }
            uint32_t *dst = sA + (lr + 64 * i) * A_PITCH + 8 * lq;
            *(uint4 *)dst = make_uint4(c[0], c[1], c[2], c[3]);
            *(uint4 *)(dst + 4) = make_uint4(c[4], c[5], c[6], c[7]);
        }
#pragma unroll
        for (int i = 0; i < WN; ++i) {
            bsum[i] += __popc(pw[i].x) + __popc(pw[i].y) + __popc(pw[i].z) + __popc(pw[i].w);
            uint32_t *dst = sW + (lr + 64 * i) * W_PITCH + 4 * lq;
            *(uint2 *)dst = make_uint2(pw[i].x, pw[i].y);
            *(uint2 *)(dst + 2) = make_uint2(pw[i].z, pw[i].w);
        }
    };

    v16i acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    fetch(0);
    stage(0);
    __syncthreads();

    int buf = 0;
    for (int k0 = 0; k0 < rw; k0 += KT) {
        const bool more = k0 + KT < rw;
        if (more) fetch(k0 + KT);

        const uint32_t *sA = smem + buf * T::BUF_DWORDS;
        const uint32_t *sW = sA + T::BM * A_PITCH;
        const int nblk = (rw - k0 >= KT) ? 4 : (rw - k0) / 4;  // 128-k blocks present in this step
        for (int blk = 0; blk < nblk; ++blk) {
            uint4 ua[WM];
            uint2 xw[WN];
#pragma unroll
            for (int i = 0; i < WM; ++i)
                ua[i] = *(const uint4 *)(sA + (wm * 32 * WM + 32 * i + r32) * A_PITCH + 8 * blk + 4 * h);
#pragma unroll
            for (int j = 0; j < WN; ++j)
                xw[j] = *(const uint2 *)(sW + (wn * 32 * WN + 32 * j + r32) * W_PITCH + 4 * blk + 2 * h);
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                v4i a[WM], b[WN];
#pragma unroll
                for (int i = 0; i < WM; ++i) {
                    const uint32_t u = s == 0 ? ua[i].x : s == 1 ? ua[i].y : s == 2 ? ua[i].z : ua[i].w;
                    a[i] = widen_act(u);
                }
#pragma unroll
                for (int j = 0; j < WN; ++j) {
                    const uint32_t x = s < 2 ? xw[j].x : xw[j].y;
                    b[j] = (s & 1) ? widen_w_odd(x) : widen_w_even(x);
                }
#pragma unroll
                for (int i = 0; i < WM; ++i)
#pragma unroll
                    for (int j = 0; j < WN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i][j], 0, 0, 0);
            }
        }

        if (more) stage(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }

    // row / column sums collected by the loader threads: 4 threads share a row
#pragma unroll
    for (int i = 0; i < WM; ++i) {
        int v = tsum[i];
        v += __shfl_xor(v, 1);
        v += __shfl_xor(v, 2);
        if (lq == 0) sT[lr + 64 * i] = v;
    }
#pragma unroll
    for (int i = 0; i < WN; ++i) {
        int v = bsum[i];
        v += __shfl_xor(v, 1);
        v += __shfl_xor(v, 2);
        if (lq == 0) sB[lr + 64 * i] = v;
    }
    __syncthreads();

    // epilogue; the tile buffers are dead (last loop barrier), sT / sB live behind them
    float *sa_lds = (float *)smem;
    uint16_t *strip = (uint16_t *)(smem + T::BM) + wave * (32 * (32 * WN + 8));
    for (int t = tid; t < T::BM; t += 256) sa_lds[t] = (m0 + t < g.M) ? load_scale(g.s_a, m0 + t) : 0.0f;
    __syncthreads();
    int b2[WN];
#pragma unroll
    for (int j = 0; j < WN; ++j) b2[j] = 2 * sB[wn * 32 * WN + 32 * j + r32];
    store_wave_tile<WM, WN>(g, m0 + wm * WM * 32, n0 + wn * WN * 32, wm * WM * 32, strip, sa_lds,
                            [&](int i, int j, int v) {
                                const int ml = wm * 32 * WM + 32 * i + 8 * (v >> 2) + 4 * h + (v & 3);
                                return sT[ml] + b2[j] - (acc[i][j][v] >> 4);
                            });
}

template <int WM, int WN>
hipError_t launch(const GemmArgs &g, hipStream_t st)
{
    using T = Tile<WM, WN>;
    static bool configured = false;  // benign race: the attribute is idempotent
    if (!configured) {
        hipError_t e = hipFuncSetAttribute((const void *)k_gemm_mfma<WM, WN>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, T::SMEM_BYTES);
        if (e != hipSuccess) return e;
        configured = true;
    }
    dim3 grid((g.N + T::BN - 1) / T::BN, (g.M + T::BM - 1) / T::BM);
    hipLaunchKernelGGL((k_gemm_mfma<WM, WN>), grid, dim3(256), T::SMEM_BYTES, st, g);
    return hipGetLastError();
}

}  // namespace

bool gemm_mfma_supported(const GemmArgs &g) { return g.M > 0 && g.N > 0 && g.rw > 0; }

hipError_t launch_gemm_mfma(const GemmArgs &g, hipStream_t st)
{
    // Largest tile that still gives every compute unit work (256 CUs).
    auto tiles = [&](int bm, int bn) { return (int64_t)((g.M + bm - 1) / bm) * ((g.N + bn - 1) / bn); };
    if (tiles(256, 256) >= 384) return launch<4, 4>(g, st);
    if (tiles(128, 256) >= 256) return launch<2, 4>(g, st);
    return launch<2, 2>(g, st);
}

}  // namespace bwta
