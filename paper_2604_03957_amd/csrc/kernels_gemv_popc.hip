// Decode-shaped BWTA product (a handful of tokens against a large weight matrix): the packed
// weights are streamed from HBM exactly once with 128-bit loads, the few activation rows live in
// registers, and each weight word costs one three-input boolean op plus one popcount-accumulate
// per token:  acc = popc(mask) - 2 * popc(mask & (sign ^ wsign))   (Case 1, xor form).
//
// A weight row of C4 16-byte chunks is spread over G lanes (chunk c -> lane c % G, slot c / G), so
// the G lanes of a group read G * 16 contiguous bytes per slot and 64 / G rows share a wavefront.
// Lane partial counts are summed across the group with DPP adds, then the group's lanes write one
// token each.  One launch can walk several problems of the same shape (grid.y), which is how a
// decode step's independent matrices (or a bandwidth measurement) share one dispatch.
#include "bwta_internal.h"

namespace bwta {

namespace {

__device__ __forceinline__ int popc4(const uint4 &m, const uint4 &s, const uint4 &w)
{
    return __popc(m.x & (s.x ^ w.x)) + __popc(m.y & (s.y ^ w.y)) + __popc(m.z & (s.z ^ w.z)) +
           __popc(m.w & (s.w ^ w.w));
}

// sum over the G lanes of a group (G = 8, 16, 32 or 64 consecutive lanes); every lane gets the sum
template <int G>
__device__ __forceinline__ int group_sum(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0xb1, 0xf, 0xf, true);   // quad_perm [1,0,3,2]
    v += __builtin_amdgcn_update_dpp(0, v, 0x4e, 0xf, 0xf, true);   // quad_perm [2,3,0,1]
    v += __builtin_amdgcn_update_dpp(0, v, 0x141, 0xf, 0xf, true);  // row_half_mirror: lane i <-> 7 - i
    if (G >= 16) v += __builtin_amdgcn_update_dpp(0, v, 0x140, 0xf, 0xf, true);  // row_mirror: i <-> 15 - i
    if (G >= 32) v += __shfl_xor(v, 16);
    if (G >= 64) v += __shfl_xor(v, 32);
    return v;
}

struct GemvBatch {
    static constexpr int MAX = 32;
    const uint32_t *mask[MAX], *sign[MAX], *wsign[MAX];
    const uint16_t *s_a[MAX], *s_w[MAX];
    int32_t *acc[MAX];
    uint16_t *out[MAX];
};

struct GemvShape {
    int M, N, rw, C4, a_mode, w_mode;
    int64_t ldo;
};

template <int MT, int G, int NCH, int UNR>
__global__ __launch_bounds__(256) void k_gemv_popc(GemvBatch b, GemvShape sh)
{
    const int lane = threadIdx.x & 63;
    const int gw = blockIdx.x * 4 + (threadIdx.x >> 6);  // wavefront id within the problem
    const int p = blockIdx.y;
    constexpr int RPP = 64 / G;  // rows per pass of one wavefront
    const int sub = lane / G, cl = lane % G;
    const int rw = sh.rw;
    const uint4 zero4 = make_uint4(0, 0, 0, 0);
    const uint32_t *mask = b.mask[p], *sign = b.sign[p], *wsign = b.wsign[p];

    bool valid[NCH];
#pragma unroll
    for (int j = 0; j < NCH; ++j) valid[j] = cl + G * j < sh.C4;

    // this wavefront's weight rows: UNR passes, issued first (HBM latency), before the cache-resident activations
    const int64_t row0 = ((int64_t)gw * UNR) * RPP + sub;
    uint4 w[UNR][NCH];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
        const int64_t n = row0 + (int64_t)u * RPP;
#pragma unroll
        for (int j = 0; j < NCH; ++j) {
            w[u][j] = zero4;
            if (n < sh.N && valid[j]) w[u][j] = *(const uint4 *)(wsign + n * rw + 4 * (cl + G * j));
        }
    }

    // activation rows -> registers (tiny, cache resident)
    uint4 am[MT][NCH], as[MT][NCH];
    int nnz[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        int c = 0;
#pragma unroll
        for (int j = 0; j < NCH; ++j) {
            am[m][j] = zero4;
            as[m][j] = zero4;
            if (m < sh.M && valid[j]) {
                am[m][j] = *(const uint4 *)(mask + (int64_t)m * rw + 4 * (cl + G * j));
                as[m][j] = *(const uint4 *)(sign + (int64_t)m * rw + 4 * (cl + G * j));
            }
            c += __popc(am[m][j].x) + __popc(am[m][j].y) + __popc(am[m][j].z) + __popc(am[m][j].w);
        }
        nnz[m] = group_sum<G>(c);
    }

    const ScaleArg sa{b.s_a[p], b.s_a[p] ? sh.a_mode : 0}, sw{b.s_w[p], b.s_w[p] ? sh.w_mode : 0};
    int32_t *acc = b.acc[p];
    uint16_t *out = b.out[p];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
        const int64_t n = row0 + (int64_t)u * RPP;
        int cnt[MT];
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            int c = 0;
#pragma unroll
            for (int j = 0; j < NCH; ++j) c += popc4(am[m][j], as[m][j], w[u][j]);
            cnt[m] = group_sum<G>(c);
        }
        if (n >= sh.N) continue;
        const float swv = load_scale(sw, (int)n);
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            if (m < sh.M && m == cl) {  // lane m of the group writes token m (G >= 8 >= MT)
                const int a = nnz[m] - 2 * cnt[m];
                if (acc) acc[(int64_t)m * sh.N + n] = a;
                if (out) out[(int64_t)m * sh.ldo + n] = scaled_to_half(a, load_scale(sa, m) * swv);
            }
        }
    }
}

template <int MT, int G, int NCH>
hipError_t launch_t(const GemvBatch &b, int count, const GemvShape &sh, hipStream_t st)
{
    // passes in flight per wavefront: as many as fit next to the activation rows in ~190 registers
    constexpr int ROOM = (190 - MT * NCH * 8) / (4 * NCH);
    constexpr int UNR = ROOM >= 4 ? 4 : (ROOM >= 2 ? 2 : 1);
    constexpr int RPP = 64 / G;
    const int64_t passes = ((int64_t)sh.N + RPP - 1) / RPP;
    const int64_t waves = (passes + UNR - 1) / UNR;
    const unsigned grid = (unsigned)((waves + 3) / 4);
    hipLaunchKernelGGL((k_gemv_popc<MT, G, NCH, UNR>), dim3(grid, count), dim3(256), 0, st, b, sh);
    return hipGetLastError();
}

template <int MT>
hipError_t launch_m(const GemvBatch &b, int count, const GemvShape &sh, hipStream_t st)
{
    // smallest group that keeps the activation rows within ~128 registers: MT * NCH <= 16
    const int C4 = sh.C4;
    constexpr int CAP = 16 / MT;  // chunks per lane allowed
#define BWTA_GEMV_TRY(G_, NCH_)                                                    \
    if constexpr (NCH_ <= CAP) {                                                  \
        if (C4 <= G_ * NCH_) return launch_t<MT, G_, NCH_>(b, count, sh, st);     \
    }
    BWTA_GEMV_TRY(8, 1)
    BWTA_GEMV_TRY(8, 2)
    BWTA_GEMV_TRY(8, 4)
    BWTA_GEMV_TRY(16, 4)
    BWTA_GEMV_TRY(8, 11)
    BWTA_GEMV_TRY(8, 16)
    BWTA_GEMV_TRY(16, 2)
    BWTA_GEMV_TRY(16, 6)
    BWTA_GEMV_TRY(16, 8)
    BWTA_GEMV_TRY(32, 1)
    BWTA_GEMV_TRY(32, 2)
    BWTA_GEMV_TRY(32, 3)
    BWTA_GEMV_TRY(32, 4)
    BWTA_GEMV_TRY(64, 1)
    BWTA_GEMV_TRY(64, 2)
#undef BWTA_GEMV_TRY
    return hipErrorInvalidValue;
}

hipError_t launch_any(const GemvBatch &b, int count, const GemvShape &sh, hipStream_t st)
{
    if (sh.M <= 1) return launch_m<1>(b, count, sh, st);
    if (sh.M <= 2) return launch_m<2>(b, count, sh, st);
    if (sh.M <= 4) return launch_m<4>(b, count, sh, st);
    return launch_m<8>(b, count, sh, st);
}

}  // namespace

// M <= 8 tokens and K <= 16384 (at most two 16-byte chunks per lane at the widest group).
bool gemv_popc_supported(const GemmArgs &g) { return g.M >= 1 && g.M <= 8 && g.rw / 4 <= 128 && g.N >= 1; }

hipError_t launch_gemv_popc(const GemmArgs &g, hipStream_t st)
{
    GemvBatch b;
    b.mask[0] = g.mask; b.sign[0] = g.sign; b.wsign[0] = g.wsign;
    b.s_a[0] = g.s_a.mode ? g.s_a.ptr : nullptr;
    b.s_w[0] = g.s_w.mode ? g.s_w.ptr : nullptr;
    b.acc[0] = g.acc; b.out[0] = g.out;
    GemvShape sh{g.M, g.N, g.rw, g.rw / 4, g.s_a.mode, g.s_w.mode, g.ldo};
    return launch_any(b, 1, sh, st);
}

// count problems of one shape; pointers given as host arrays of device pointers
hipError_t launch_gemv_popc_grouped(const GemmArgs *gs, int count, hipStream_t st)
{
    for (int base = 0; base < count; base += GemvBatch::MAX) {
        const int n = count - base < GemvBatch::MAX ? count - base : GemvBatch::MAX;
        GemvBatch b;
        for (int i = 0; i < n; ++i) {
            const GemmArgs &g = gs[base + i];
            b.mask[i] = g.mask; b.sign[i] = g.sign; b.wsign[i] = g.wsign;
            b.s_a[i] = g.s_a.mode ? g.s_a.ptr : nullptr;
            b.s_w[i] = g.s_w.mode ? g.s_w.ptr : nullptr;
            b.acc[i] = g.acc; b.out[i] = g.out;
        }
        const GemmArgs &g0 = gs[base];
        GemvShape sh{g0.M, g0.N, g0.rw, g0.rw / 4, g0.s_a.mode, g0.s_w.mode, g0.ldo};
        hipError_t e = launch_any(b, n, sh, st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace bwta
