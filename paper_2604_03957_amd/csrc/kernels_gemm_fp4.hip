// BWTA product on the FP4 matrix cores (v_mfma_f32_32x32x64_f8f6f4, both operands E2M1).
//
// +1, -1 and 0 are exact E2M1 values (0b0010, 0b1010, 0b0000) and every partial sum is an
// integer below 2^24, so the fp32 accumulators hold the exact BWTA product (Case 1 of the
// paper's arithmetic rules) while the instruction retires twice the MACs of the int8 form.
//   * Activations are converted once per call from the two bit planes into E2M1 nibbles
//     (bit 1 = mask, bit 3 = sign) in a fragment-major layout: [row block of 32][k step of
//     64][lane][4 dwords], so a wavefront's operand is one contiguous kilobyte.
//   * Weights stay one bit each in HBM and LDS; a lane widens the 32 bits it needs for one
//     instruction into four dwords of nibbles with three shifts and four and-or ops.
// The dot product does not depend on the order of k inside an instruction, so element
// 4 i + d of a 32-bit word goes to nibble i of dword d in BOTH operands, which is what makes
// the widening that cheap.
#include "bwta_internal.h"

namespace bwta {

namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int W_PITCH = 12;  // dwords per LDS weight row: 8 words of a 256-k chunk + 4 pad

// Which k step and lane half consume plane word q (identical rule in the converter and the GEMM):
// words are taken in groups of 8 (one 256-k chunk); word j of a group feeds step 2*(j/4) + j%2
// of the chunk on lane half (j%4)/2.
__device__ __forceinline__ void word_slot(int q, int &step, int &half)
{
    const int c = q >> 3, j = q & 7;
    step = 4 * c + 2 * (j >> 2) + (j & 1);
    half = (j & 3) >> 1;
}

// planes -> E2M1 fragments.  One thread per (row, 4 words): 128-bit plane loads, and the 32 rows
// of a row block sit on consecutive lanes so every 16-byte fragment store is part of a
// contiguous 512-byte run.
__global__ __launch_bounds__(256) void k_planes_to_fp4(const uint32_t *__restrict__ mask,
                                                       const uint32_t *__restrict__ sign, int M, int rw,
                                                       int rows_padded, uint32_t *__restrict__ frag)
{
    const int rw4 = rw >> 2;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t total = (int64_t)rows_padded * rw4;
    if (gid >= total) return;
    const int r = (int)(gid & 31);
    const int64_t rest = gid >> 5;
    const int q4 = (int)(rest % rw4);
    const int rb = (int)(rest / rw4);
    const int m = rb * 32 + r;
    uint4 mk4 = make_uint4(0, 0, 0, 0), sg4 = mk4;
    if (m < M) {
        mk4 = *(const uint4 *)(mask + (int64_t)m * rw + 4 * q4);
        sg4 = *(const uint4 *)(sign + (int64_t)m * rw + 4 * q4);
    }
    const uint32_t mks[4] = {mk4.x, mk4.y, mk4.z, mk4.w};
    const uint32_t sgs[4] = {sg4.x, sg4.y, sg4.z, sg4.w};
    const int S = rw / 2;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const uint32_t mk = mks[w], sg = sgs[w] & mk;
        uint4 o;
        o.x = ((sg << 3) & 0x88888888u) | ((mk << 1) & 0x22222222u);
        o.y = ((sg << 2) & 0x88888888u) | (mk & 0x22222222u);
        o.z = ((sg << 1) & 0x88888888u) | ((mk >> 1) & 0x22222222u);
        o.w = (sg & 0x88888888u) | ((mk >> 2) & 0x22222222u);
        int step, half;
        word_slot(4 * q4 + w, step, half);
        *(uint4 *)(frag + (((int64_t)rb * S + step) * 64 + half * 32 + r) * 4) = o;
    }
}

// weight bits -> E2M1 nibbles (+1 = 0b0010, -1 = 0b1010): element 4 i + d -> nibble i of dword d
// m88 = 0x88888888 and c22 = 0x22222222 are passed in registers the optimiser cannot see
// through, so each dword is one v_and_or_b32 (VOP3 cannot carry two literals on this ISA).
__device__ __forceinline__ v8i widen_w(uint32_t x, uint32_t m88, uint32_t c22)
{
    v8i r;
    r[0] = (int)(((x << 3) & m88) | c22);
    r[1] = (int)(((x << 2) & m88) | c22);
    r[2] = (int)(((x << 1) & m88) | c22);
    r[3] = (int)((x & m88) | c22);
    r[4] = r[5] = r[6] = r[7] = 0;
    return r;
}

template <int WM, int WN, int WAVES_M, int WAVES_N>
struct Cfg {
    static constexpr int BM = 32 * WM * WAVES_M, BN = 32 * WN * WAVES_N;
    static constexpr int THREADS = 64 * WAVES_M * WAVES_N;
    static constexpr int A_DW = (BM / 32) * 1024;  // 4 steps * 64 lanes * 4 dwords per row block
    static constexpr int W_DW = BN * W_PITCH;
    static constexpr int BUF_DW = A_DW + W_DW;
    static constexpr int EPI_BYTES = BM * 4 + (THREADS / 64) * 32 * (32 * WN + 8) * 2;
    static constexpr int SMEM_BYTES = 2 * BUF_DW * 4 > EPI_BYTES ? 2 * BUF_DW * 4 : EPI_BYTES;
    static constexpr int A_PIECES = (BM / 32) * 256;  // 16-byte pieces per chunk
    static constexpr int W_PIECES = BN * 2;
    static constexpr int A_LOADS = (A_PIECES + THREADS - 1) / THREADS;
    static constexpr int W_LOADS = (W_PIECES + THREADS - 1) / THREADS;
};

template <int WM, int WN, int WAVES_M, int WAVES_N>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N)
__attribute__((amdgpu_waves_per_eu(WM * WN >= 16 ? 1 : 2, WM * WN >= 16 ? 1 : 2))) void k_gemm_fp4(GemmArgs g, const uint32_t *__restrict__ frag,
                                                                     int row_blocks)
{
    using C = Cfg<WM, WN, WAVES_M, WAVES_N>;
    extern __shared__ __attribute__((aligned(16))) uint32_t smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int r32 = lane & 31, h = lane >> 5;
    const int m0 = blockIdx.y * C::BM, n0 = blockIdx.x * C::BN;
    const int rb0 = blockIdx.y * (C::BM / 32);
    const int rw = g.rw, S = rw / 2;
    const int nchunks = (rw + 7) / 8;

    uint32_t m88 = 0x88888888u, c22 = 0x22222222u;
    asm volatile("" : "+s"(m88));
    asm volatile("" : "+v"(c22));

    uint4 pa[C::A_LOADS], pw[C::W_LOADS];

    auto fetch = [&](int c) {
#pragma unroll
        for (int i = 0; i < C::A_LOADS; ++i) {
            const int p = tid + i * C::THREADS;  // piece: row block p/256, step (p%256)/64, lane p%64
            const int rb = rb0 + (p >> 8), step = 4 * c + ((p >> 6) & 3);
            pa[i] = make_uint4(0, 0, 0, 0);
            if (p < C::A_PIECES && rb < row_blocks && step < S)
                pa[i] = *(const uint4 *)(frag + (((int64_t)rb * S + step) * 64 + (p & 63)) * 4);
        }
#pragma unroll
        for (int i = 0; i < C::W_LOADS; ++i) {
            const int p = tid + i * C::THREADS;  // piece: row p/2, half p%2
            const int n = n0 + (p >> 1), kw = 8 * c + 4 * (p & 1);
            pw[i] = make_uint4(0, 0, 0, 0);
            if (p < C::W_PIECES && n < g.N && kw < rw) pw[i] = *(const uint4 *)(g.wsign + (int64_t)n * rw + kw);
        }
    };

    auto stage = [&](int buf) {
        uint32_t *sA = smem + buf * C::BUF_DW;
        uint32_t *sW = sA + C::A_DW;
#pragma unroll
        for (int i = 0; i < C::A_LOADS; ++i) {
            const int p = tid + i * C::THREADS;
            if (p < C::A_PIECES) *(uint4 *)(sA + 4 * p) = pa[i];
        }
#pragma unroll
        for (int i = 0; i < C::W_LOADS; ++i) {
            const int p = tid + i * C::THREADS;
            if (p < C::W_PIECES) {
                // chunk words w0..w7 are stored as [w0 w1 w4 w5 | w2 w3 w6 w7] so that lane half h
                // finds the words of steps 0..3 in one 16-byte read at 4 h
                uint32_t *row = sW + (p >> 1) * W_PITCH;
                const int half = p & 1;
                *(uint2 *)(row + 2 * half) = make_uint2(pw[i].x, pw[i].y);
                *(uint2 *)(row + 4 + 2 * half) = make_uint2(pw[i].z, pw[i].w);
            }
        }
    };

    v16f acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    fetch(0);
    stage(0);
    __syncthreads();

    int buf = 0;
    for (int c = 0; c < nchunks; ++c) {
        const bool more = c + 1 < nchunks;
        if (more) fetch(c + 1);

        const uint32_t *sA = smem + buf * C::BUF_DW;
        const uint32_t *sW = sA + C::A_DW;
        // always four steps: a short last chunk was staged with zeros, which add nothing
        uint4 xw[WN];
#pragma unroll
        for (int j = 0; j < WN; ++j)
            xw[j] = *(const uint4 *)(sW + ((wn * WN + j) * 32 + r32) * W_PITCH + 4 * h);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            {
                v8i a[WM], b[WN];
#pragma unroll
                for (int i = 0; i < WM; ++i) {
                    const uint4 u = *(const uint4 *)(sA + (((wm * WM + i) * 4 + s) * 64 + lane) * 4);
                    a[i][0] = (int)u.x; a[i][1] = (int)u.y; a[i][2] = (int)u.z; a[i][3] = (int)u.w;
                    a[i][4] = a[i][5] = a[i][6] = a[i][7] = 0;
                }
#pragma unroll
                for (int j = 0; j < WN; ++j)
                    b[j] = widen_w(s == 0 ? xw[j].x : s == 1 ? xw[j].y : s == 2 ? xw[j].z : xw[j].w, m88, c22);
#pragma unroll
                for (int i = 0; i < WM; ++i)
#pragma unroll
                    for (int j = 0; j < WN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[i], b[j], acc[i][j], 4, 4, 0,
                                                                                    0, 0, 0);
            }
        }

        if (more) stage(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }

    // epilogue (the loop's last barrier has retired every LDS read, so the tiles can be reused)
    float *sa_lds = (float *)smem;
    uint16_t *strip = (uint16_t *)(smem + C::BM) + wave * (32 * (32 * WN + 8));
    for (int t = tid; t < C::BM; t += C::THREADS) sa_lds[t] = (m0 + t < g.M) ? load_scale(g.s_a, m0 + t) : 0.0f;
    __syncthreads();
    store_wave_tile<WM, WN>(g, m0 + wm * WM * 32, n0 + wn * WN * 32, wm * WM * 32, strip, sa_lds,
                            [&](int i, int j, int v) { return (int)acc[i][j][v]; });
}

template <int WM, int WN, int WAVES_M, int WAVES_N>
hipError_t launch(const GemmArgs &g, const uint32_t *frag, hipStream_t st)
{
    using C = Cfg<WM, WN, WAVES_M, WAVES_N>;
    static bool configured = false;  // benign race: setting the attribute twice is harmless
    if (!configured) {
        hipError_t e = hipFuncSetAttribute((const void *)k_gemm_fp4<WM, WN, WAVES_M, WAVES_N>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, C::SMEM_BYTES);
        if (e != hipSuccess) return e;
        configured = true;
    }
    dim3 grid((g.N + C::BN - 1) / C::BN, (g.M + C::BM - 1) / C::BM);
    hipLaunchKernelGGL((k_gemm_fp4<WM, WN, WAVES_M, WAVES_N>), grid, dim3(C::THREADS), C::SMEM_BYTES, st, g, frag,
                       (g.M + 31) / 32);
    return hipGetLastError();
}

}  // namespace

size_t gemm_fp4_frag_bytes(int M, int K)
{
    const size_t rw = 4 * (((size_t)K + 127) / 128);
    return (size_t)((M + 31) / 32) * 32 * rw * 16;  // 4 bits per element of the padded matrix
}

hipError_t launch_gemm_fp4(const GemmArgs &g, uint32_t *frag, hipStream_t st)
{
    const int rows_padded = (g.M + 31) / 32 * 32;
    const int64_t total = (int64_t)rows_padded * (g.rw / 4);
    hipLaunchKernelGGL(k_planes_to_fp4, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, g.mask, g.sign,
                       g.M, g.rw, rows_padded, frag);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    auto tiles = [&](int bm, int bn) { return (int64_t)((g.M + bm - 1) / bm) * ((g.N + bn - 1) / bn); };
    if (tiles(128, 256) >= 512) return launch<2, 4, 2, 2>(g, frag, st);
    return launch<2, 2, 2, 2>(g, frag, st);
}

}  // namespace bwta
