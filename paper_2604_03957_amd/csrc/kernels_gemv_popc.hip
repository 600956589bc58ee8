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
#include <atomic>

#include "bwta_internal.h"

namespace bwta {

namespace {

// acc + popc(x): v_bcnt_u32_b32 accumulates for free; spelled out so the adds are not re-associated
// into separate v_add3 instructions
__device__ __forceinline__ int popc_acc(uint32_t x, int acc)
{
    int r;
    asm("v_bcnt_u32_b32 %0, %1, %2" : "=v"(r) : "v"(x), "v"(acc));
    return r;
}

__device__ __forceinline__ int popc4(const uint4 &m, const uint4 &s, const uint4 &w, int acc)
{
    acc = popc_acc(m.x & (s.x ^ w.x), acc);
    acc = popc_acc(m.y & (s.y ^ w.y), acc);
    acc = popc_acc(m.z & (s.z ^ w.z), acc);
    return popc_acc(m.w & (s.w ^ w.w), acc);
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

typedef unsigned v4u_t __attribute__((ext_vector_type(4)));

struct GemvBatch {
    static constexpr int MAX = 64;
    const uint32_t *mask[MAX], *sign[MAX], *wsign[MAX];
    const uint16_t *s_a[MAX], *s_w[MAX];
    int32_t *acc[MAX];
    uint16_t *out[MAX];
};

struct GemvShape {
    int M, N, rw, C4, a_mode, w_mode;
    int64_t ldo;
};

template <int MT, int G, int NCH, int UNR, bool NT>
__global__ __launch_bounds__(256) void k_gemv_popc(GemvBatch b, GemvShape sh)
{
    const int lane = threadIdx.x & 63;
    const int gw = blockIdx.x * 4 + (threadIdx.x >> 6);  // wavefront id within the problem
    const int p = blockIdx.y;
    constexpr int RPP = 64 / G;  // rows per pass of one wavefront
    const int sub = lane / G, cl = lane % G;
    const int rw = sh.rw;
    const uint32_t *mask = b.mask[p], *sign = b.sign[p], *wsign = b.wsign[p];

    // chunk j of this lane is cl + G j.  Chunks past the row end are clamped to the last chunk for
    // the weight loads (never predicated) and get all-zero activation masks, so they add nothing.
    int coff[NCH];  // dword offset of chunk j inside a row
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
        const int c = cl + G * j;
        coff[j] = 4 * (c < sh.C4 ? c : sh.C4 - 1);
    }

    // Request order: the scales the epilogue needs, the activation rows (small, cache-resident), then
    // the weight rows of all UNR passes.  Memory returns in request order, so the activations can be
    // parked in LDS while the weights are still in flight, each pass waits for its own rows only,
    // and the end of the kernel waits for no load at all.  Every lane issues every load (a lane with
    // nothing to fetch reads the matrix's first bytes and drops them), so no wait hides in a branch.
    const ScaleArg sa{b.s_a[p], b.s_a[p] ? sh.a_mode : 0}, sw{b.s_w[p], b.s_w[p] ? sh.w_mode : 0};
    const bool writer = cl < sh.M;  // lane cl of a group writes token cl (G >= 8 >= MT)
    const uint16_t *safe = (const uint16_t *)wsign;
    const int64_t row0 = ((int64_t)gw * UNR) * RPP + sub;
    const uint16_t sa_raw = *((sa.mode && writer) ? sa.ptr + (sa.mode == 1 ? 0 : cl) : safe);
    uint16_t sw_raw[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
        int64_t n = row0 + (int64_t)u * RPP;
        n = n < sh.N ? n : sh.N - 1;
        sw_raw[u] = *(sw.mode ? sw.ptr + (sw.mode == 1 ? 0 : n) : safe);
    }

    // activation rows: staged once per workgroup in LDS (coalesced), then each lane keeps the
    // chunks it needs in registers.  Layout: [token][plane][chunk] of 16 bytes.
    extern __shared__ __attribute__((aligned(16))) uint4 s_act[];
    constexpr int NSTAGE = (MT * 2 * G * NCH + 255) / 256;  // staging loads per thread
    constexpr bool EARLY = NSTAGE <= 2;  // more rows than that are staged by a loop behind the weights
    constexpr int NST = EARLY ? NSTAGE : 0;
    const int act_pieces = sh.M * 2 * sh.C4;
    uint4 stage[NST > 0 ? NST : 1];
#pragma unroll
    for (int k = 0; k < NST; ++k) {
        const int idx = threadIdx.x + 256 * k;
        const int ic = idx < act_pieces ? idx : 0;
        const int c = ic % sh.C4, pl = (ic / sh.C4) & 1, m = ic / (2 * sh.C4);
        stage[k] = *(const uint4 *)((pl ? sign : mask) + (int64_t)m * rw + 4 * c);
    }

    // weight rows of this wavefront: UNR passes; rows past N are clamped to the last row and never
    // stored.  Rows that are whole 128-byte lines are streamed past the caches (NT).
    uint4 w[UNR][NCH];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
        int64_t n = row0 + (int64_t)u * RPP;
        n = n < sh.N ? n : sh.N - 1;
        const uint32_t *wrow = wsign + n * rw;
#pragma unroll
        for (int j = 0; j < NCH; ++j) {
            const v4u_t *src = (const v4u_t *)(wrow + coff[j]);
            const v4u_t x = NT ? __builtin_nontemporal_load(src) : *src;
            w[u][j] = make_uint4(x[0], x[1], x[2], x[3]);
        }
    }
    __builtin_amdgcn_sched_barrier(0);  // nothing above is waited for before every request is out

#pragma unroll
    for (int k = 0; k < NST; ++k) {
        const int idx = threadIdx.x + 256 * k;
        if (idx < act_pieces) s_act[idx] = stage[k];
    }
    if (!EARLY) {
        for (int idx = threadIdx.x; idx < act_pieces; idx += 256) {
            const int c = idx % sh.C4, pl = (idx / sh.C4) & 1, m = idx / (2 * sh.C4);
            s_act[idx] = *(const uint4 *)((pl ? sign : mask) + (int64_t)m * rw + 4 * c);
        }
    }
    __syncthreads();
    const uint4 zero4 = make_uint4(0, 0, 0, 0);
    uint4 am[MT][NCH], as[MT][NCH];
    int my_nnz = 0;  // nnz of token cl (the token this lane writes)
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        int c = 0;
#pragma unroll
        for (int j = 0; j < NCH; ++j) {
            const bool live = (m < sh.M) && (cl + G * j < sh.C4);
            am[m][j] = live ? s_act[(2 * m) * sh.C4 + (coff[j] >> 2)] : zero4;
            as[m][j] = s_act[(m < sh.M ? 2 * m + 1 : 1) * sh.C4 + (coff[j] >> 2)];
            c = popc_acc(am[m][j].x, popc_acc(am[m][j].y, popc_acc(am[m][j].z, popc_acc(am[m][j].w, c))));
        }
        c = group_sum<G>(c);
        my_nnz = (cl == m) ? c : my_nnz;
    }

    int32_t *acc = b.acc[p];
    uint16_t *out = b.out[p];
    const float my_sa = (sa.mode && writer) ? half_bits_to_float(sa_raw) : 1.0f;
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
        const int64_t n = row0 + (int64_t)u * RPP;
        int my_cnt = 0;
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            int c = 0;
#pragma unroll
            for (int j = 0; j < NCH; ++j) c = popc4(am[m][j], as[m][j], w[u][j], c);
            c = group_sum<G>(c);
            my_cnt = (cl == m) ? c : my_cnt;
        }
        if (writer && n < sh.N) {
            const int a = my_nnz - 2 * my_cnt;
            if (acc) acc[(int64_t)cl * sh.N + n] = a;
            const float my_sw = sw.mode ? half_bits_to_float(sw_raw[u]) : 1.0f;
            if (out) out[(int64_t)cl * sh.ldo + n] = scaled_to_half(a, my_sa * my_sw);
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
    const size_t lds = (size_t)sh.M * 2 * sh.C4 * 16;  // <= 8 * 2 * 128 * 16 = 32 KiB
    const bool nt = (sh.rw & 31) == 0;
    // A single small matrix: one pass per wavefront, so that every compute unit gets a workgroup
    // (with 4 passes a 4096-row matrix is 128 workgroups for 256 compute units).
    if constexpr (MT <= 2 && UNR > 1) {
        if (((passes + UNR - 1) / UNR + 3) / 4 * count < 512) {
            const unsigned grid1 = (unsigned)((passes + 3) / 4);
            if (nt)
                hipLaunchKernelGGL((k_gemv_popc<MT, G, NCH, 1, true>), dim3(grid1, count), dim3(256), lds, st, b, sh);
            else
                hipLaunchKernelGGL((k_gemv_popc<MT, G, NCH, 1, false>), dim3(grid1, count), dim3(256), lds, st, b, sh);
            return hipGetLastError();
        }
    }
    const int64_t waves = (passes + UNR - 1) / UNR;
    const unsigned grid = (unsigned)((waves + 3) / 4);
    if (nt)
        hipLaunchKernelGGL((k_gemv_popc<MT, G, NCH, UNR, true>), dim3(grid, count), dim3(256), lds, st, b, sh);
    else
        hipLaunchKernelGGL((k_gemv_popc<MT, G, NCH, UNR, false>), dim3(grid, count), dim3(256), lds, st, b, sh);
    return hipGetLastError();
}

std::atomic<int> g_force_g{0}, g_force_nch{0};  // tuning override (bwta_set_tile; relaxed: a launch sees old or new)

template <int MT>
hipError_t launch_m(const GemvBatch &b, int count, const GemvShape &sh, hipStream_t st)
{
    const int f_g = g_force_g.load(std::memory_order_relaxed), f_nch = g_force_nch.load(std::memory_order_relaxed);
#define BWTA_GEMV_FORCE(G_, NCH_)                                                                  \
    if constexpr (MT * NCH_ <= 16) {                                                               \
        if (f_g == G_ && f_nch == NCH_ && sh.C4 <= G_ * NCH_)                                      \
            return launch_t<MT, G_, NCH_>(b, count, sh, st);                                       \
    }
    BWTA_GEMV_FORCE(8, 4) BWTA_GEMV_FORCE(16, 2) BWTA_GEMV_FORCE(32, 1) BWTA_GEMV_FORCE(16, 6)
    BWTA_GEMV_FORCE(32, 3) BWTA_GEMV_FORCE(8, 11) BWTA_GEMV_FORCE(16, 4) BWTA_GEMV_FORCE(32, 2)
    BWTA_GEMV_FORCE(32, 4)
#undef BWTA_GEMV_FORCE
    // Measured on MI355X: few chunks per lane (small activation register footprint, more
    // wavefronts in flight) beats few lanes per row, so rows are spread over up to 32 lanes
    // before a lane takes a second chunk; 64 lanes only when the registers demand it.
    const int C4 = sh.C4;
    constexpr int CAP = 16 / MT;  // chunks per lane allowed (activation rows <= 128 registers)
#define BWTA_GEMV_TRY(G_, NCH_)                                                    \
    if constexpr (NCH_ <= CAP) {                                                  \
        if (C4 <= G_ * NCH_) return launch_t<MT, G_, NCH_>(b, count, sh, st);     \
    }
    BWTA_GEMV_TRY(8, 1)
    BWTA_GEMV_TRY(16, 1)
    BWTA_GEMV_TRY(32, 1)
    BWTA_GEMV_TRY(32, 2)
    BWTA_GEMV_TRY(32, 3)
    BWTA_GEMV_TRY(32, 4)
#undef BWTA_GEMV_TRY
    if constexpr (MT == 8) {  // two chunks per lane at most: the longest rows go over all 64 lanes
        if (C4 <= 128) return launch_t<MT, 64, 2>(b, count, sh, st);
    }
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

// M <= 16 tokens (more than 8 run as two token groups over the same weights) and K <= 16384
// (at most two 16-byte chunks per lane at the widest group).
bool gemv_popc_supported(const GemmArgs &g) { return g.M >= 1 && g.M <= 16 && g.rw / 4 <= 128 && g.N >= 1; }

// count problems of one shape; tokens beyond 8 become a second batch entry on the same weights
hipError_t launch_gemv_popc_grouped(const GemmArgs *gs, int count, hipStream_t st)
{
    const GemmArgs &g0 = gs[0];
    const int groups = g0.M > 8 ? 2 : 1;
    const int per_launch = GemvBatch::MAX / groups;
    for (int base = 0; base < count; base += per_launch) {
        const int n = count - base < per_launch ? count - base : per_launch;
        for (int tg = 0; tg < groups; ++tg) {  // token groups of equal size launch together
            const int m0 = 8 * tg, mt = (g0.M - m0) < 8 ? (g0.M - m0) : 8;
            GemvBatch b;
            for (int i = 0; i < n; ++i) {
                const GemmArgs &g = gs[base + i];
                b.mask[i] = g.mask + (int64_t)m0 * g.rw;
                b.sign[i] = g.sign + (int64_t)m0 * g.rw;
                b.wsign[i] = g.wsign;
                b.s_a[i] = g.s_a.mode ? g.s_a.ptr + (g.s_a.mode == 2 ? m0 : 0) : nullptr;
                b.s_w[i] = g.s_w.mode ? g.s_w.ptr : nullptr;
                b.acc[i] = g.acc ? g.acc + (int64_t)m0 * g.N : nullptr;
                b.out[i] = g.out ? g.out + (int64_t)m0 * g.ldo : nullptr;
            }
            // the call's scale modes: those of any problem that has the scale (one without reads as 1)
            int a_mode = 0, w_mode = 0;
            for (int i = 0; i < n; ++i) {
                if (gs[base + i].s_a.mode) a_mode = gs[base + i].s_a.mode;
                if (gs[base + i].s_w.mode) w_mode = gs[base + i].s_w.mode;
            }
            GemvShape sh{mt, g0.N, g0.rw, g0.rw / 4, a_mode, w_mode, g0.ldo};
            hipError_t e = launch_any(b, n, sh, st);
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

hipError_t launch_gemv_popc(const GemmArgs &g, hipStream_t st) { return launch_gemv_popc_grouped(&g, 1, st); }

void set_gemv_tile(int g, int nch)
{
    g_force_g.store(g, std::memory_order_relaxed);
    g_force_nch.store(nch, std::memory_order_relaxed);
}

}  // namespace bwta
