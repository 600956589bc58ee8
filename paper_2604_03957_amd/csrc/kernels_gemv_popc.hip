// Decode-shaped BWTA product (a handful of tokens against a large weight matrix): the packed
// weights are streamed from HBM exactly once with 128-bit loads, the few activation rows live in
// registers, and each weight word costs one three-input boolean op plus one popcount-accumulate
// per token:  acc = popc(mask) - 2 * popc(mask & (sign ^ wsign))   (Case 1, xor form).
//
// A weight row of C4 16-byte chunks is spread over G lanes (G = power of two >= min(C4, 64));
// 64/G rows share a wavefront.  Lane partial counts are summed across the group with
// cross-lane shuffles, then the group's lanes write one token each.
#include "bwta_internal.h"

namespace bwta {

namespace {

__device__ __forceinline__ int popc4(const uint4 &m, const uint4 &s, const uint4 &w)
{
    return __popc(m.x & (s.x ^ w.x)) + __popc(m.y & (s.y ^ w.y)) + __popc(m.z & (s.z ^ w.z)) +
           __popc(m.w & (s.w ^ w.w));
}

template <int MT, int NCH, int UNR>
__global__ __launch_bounds__(256) void k_gemv_popc(GemmArgs g, int G, int C4)
{
    const int lane = threadIdx.x & 63;
    const int gw = blockIdx.x * 4 + (threadIdx.x >> 6);  // global wavefront id
    const int rpp = 64 / G;                               // rows per pass of one wavefront
    const int sub = lane / G, cl = lane % G;
    const int rw = g.rw;
    const uint4 zero4 = make_uint4(0, 0, 0, 0);

    bool valid[NCH];
    int chunk[NCH];
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
        chunk[j] = cl + 64 * j;
        valid[j] = chunk[j] < C4;
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
            if (m < g.M && valid[j]) {
                am[m][j] = *(const uint4 *)(g.mask + (int64_t)m * rw + 4 * chunk[j]);
                as[m][j] = *(const uint4 *)(g.sign + (int64_t)m * rw + 4 * chunk[j]);
            }
            c += __popc(am[m][j].x) + __popc(am[m][j].y) + __popc(am[m][j].z) + __popc(am[m][j].w);
        }
        for (int off = 1; off < G; off <<= 1) c += __shfl_xor(c, off);
        nnz[m] = c;
    }

    // this wavefront's weight rows: UNR passes, all loads issued before any use
    const int64_t row0 = ((int64_t)gw * UNR) * rpp + sub;
    uint4 w[UNR][NCH];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
        const int64_t n = row0 + (int64_t)u * rpp;
#pragma unroll
        for (int j = 0; j < NCH; ++j) {
            w[u][j] = zero4;
            if (n < g.N && valid[j]) w[u][j] = *(const uint4 *)(g.wsign + n * rw + 4 * chunk[j]);
        }
    }

#pragma unroll
    for (int u = 0; u < UNR; ++u) {
        const int64_t n = row0 + (int64_t)u * rpp;
        int cnt[MT];
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            int c = 0;
#pragma unroll
            for (int j = 0; j < NCH; ++j) c += popc4(am[m][j], as[m][j], w[u][j]);
            for (int off = 1; off < G; off <<= 1) c += __shfl_xor(c, off);
            cnt[m] = c;
        }
        if (n >= g.N) continue;
        const float sw = load_scale(g.s_w, (int)n);
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            if (m < g.M && (m % G) == cl) {  // lane cl of the group writes tokens m = cl (mod G)
                const int a = nnz[m] - 2 * cnt[m];
                if (g.acc) g.acc[(int64_t)m * g.N + n] = a;
                if (g.out) g.out[(int64_t)m * g.ldo + n] = scaled_to_half(a, load_scale(g.s_a, m) * sw);
            }
        }
    }
}

template <int MT, int NCH>
hipError_t launch_t(const GemmArgs &g, int G, int C4, hipStream_t st)
{
    constexpr int UNR = (MT * NCH >= 8) ? 2 : 4;
    const int rpp = 64 / G;
    const int64_t passes = ((int64_t)g.N + rpp - 1) / rpp;
    const int64_t waves = (passes + UNR - 1) / UNR;
    const unsigned grid = (unsigned)((waves + 3) / 4);
    hipLaunchKernelGGL((k_gemv_popc<MT, NCH, UNR>), dim3(grid), dim3(256), 0, st, g, G, C4);
    return hipGetLastError();
}

}  // namespace

// M <= 8 tokens and K <= 16384 (at most two 16-byte chunks per lane).
bool gemv_popc_supported(const GemmArgs &g) { return g.M >= 1 && g.M <= 8 && g.rw / 4 <= 128 && g.N >= 1; }

hipError_t launch_gemv_popc(const GemmArgs &g, hipStream_t st)
{
    const int C4 = g.rw / 4;
    int G = 1;
    while (G < C4 && G < 64) G <<= 1;
    const int nch = C4 > 64 ? 2 : 1;
    const int mt = g.M <= 1 ? 1 : g.M <= 2 ? 2 : g.M <= 4 ? 4 : 8;
#define BWTA_GEMV_CASE(MT_, NCH_) \
    if (mt == MT_ && nch == NCH_) return launch_t<MT_, NCH_>(g, G, C4, st)
    BWTA_GEMV_CASE(1, 1);
    BWTA_GEMV_CASE(2, 1);
    BWTA_GEMV_CASE(4, 1);
    BWTA_GEMV_CASE(8, 1);
    BWTA_GEMV_CASE(1, 2);
    BWTA_GEMV_CASE(2, 2);
    BWTA_GEMV_CASE(4, 2);
    BWTA_GEMV_CASE(8, 2);
#undef BWTA_GEMV_CASE
    return hipErrorInvalidValue;
}

}  // namespace bwta
