// Pieces shared by the kernels that run the BWTA product on the FP4 matrix cores
// (v_mfma_f32_32x32x64_f8f6f4 with E2M1 operands): the 1-bit -> E2M1 widening of a weight word, the
// XCD-aware numbering of output tiles and the fp16 epilogue of a wavefront's accumulator blocks.
#pragma once
#include "bwta_internal.h"

namespace bwta {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

// weight bits -> E2M1 nibbles (+1 = 0b0010, -1 = 0b1010): element 4 i + d -> nibble i of dword d.
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

// Workgroup ids are dealt round-robin to the 8 XCDs; give every XCD a contiguous range of tile
// numbers, and number the tiles in groups of 4 token strips (strip fastest) so that the tiles an
// XCD works on at one time share both their activation strips and their weight tile in its L2.
__device__ __forceinline__ void tile_of_id(int L, int tiles_n, int tiles_total, int &tm, int &tn)
{
    const int xcd = L & 7, k = L >> 3;
    const int chunk = tiles_total >> 3, rem = tiles_total & 7;
    const int id = xcd * chunk + (xcd < rem ? xcd : rem) + k;
    const int tiles_m = tiles_total / tiles_n;
    const int per_group = 4 * tiles_n;
    const int grp = id / per_group, in_grp = id - grp * per_group;
    const int first_m = 4 * grp;
    const int gsz = tiles_m - first_m < 4 ? tiles_m - first_m : 4;
    tm = first_m + in_grp % gsz;
    tn = in_grp / gsz;
}

__device__ __forceinline__ void tile_of_workgroup(int tiles_n, int tiles_total, int &tm, int &tn)
{
    tile_of_id(blockIdx.x, tiles_n, tiles_total, tm, tn);
}

// fp16 epilogue of one wavefront: WM x WN accumulator blocks -> scaled, exactly rounded halves,
// regrouped through the wavefront's LDS strip into 16-byte row-contiguous stores.  Lane (r32, h)
// of block (j, i) holds token 32 i + r32 and channels 32 j + 8 g + 4 h + q (register 4 g + q).
// sa_w / sw_w: this wavefront's token and channel scales in LDS.
// ALPHA: the scale is fp32(alpha * (s_a * s_w)) (the attention MatMuls' prefix), else s_a * s_w (exact).
template <int WM, int WN, bool ALPHA = false>
__device__ __forceinline__ void store_tile_fp16(const v16f (&acc)[WN][WM], const GemmArgs &g, const float *sa_w,
                                                const float *sw_w, uint16_t *strip, int m_wave, int n_wave, int lane,
                                                float alpha = 1.0f)
{
    const int r32 = lane & 31, h = lane >> 5;
    constexpr int PITCH = 32 * WN + 8;  // halfs; 16-byte aligned rows, conflict-free 8-byte writes
    const bool full = (m_wave + 32 * WM <= g.M) && (n_wave + 32 * WN <= g.N) && ((g.ldo & 7) == 0) &&
                      (((uintptr_t)g.out & 15) == 0);
    // lanes per token row (8 halfs each), rows per store; with three channel blocks 60 of the 64 lanes store
    constexpr int LPR = 4 * WN, RPI = 64 / LPR;
    constexpr bool EVEN = RPI * LPR == 64 && 32 % RPI == 0;
#pragma unroll
    for (int i = 0; i < WM; ++i) {
        const float sa = sa_w[32 * i + r32];
#pragma unroll
        for (int j = 0; j < WN; ++j) {
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const int nl = 32 * j + 8 * gq + 4 * h;
                const float4 sw = *(const float4 *)(sw_w + nl);
                uint2 hv;  // four consecutive channels of this token, exactly rounded
                float f0 = sa * sw.x, f1 = sa * sw.y, f2 = sa * sw.z, f3 = sa * sw.w;
                if (ALPHA) f0 *= alpha, f1 *= alpha, f2 *= alpha, f3 *= alpha;
                hv.x = scaled_to_half2(acc[j][i][4 * gq], f0, acc[j][i][4 * gq + 1], f1);
                hv.y = scaled_to_half2(acc[j][i][4 * gq + 2], f2, acc[j][i][4 * gq + 3], f3);
                *(uint2 *)(strip + r32 * PITCH + nl) = hv;
            }
        }
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
        for (int rr = 0; rr < 32; rr += RPI) {
            const int row = rr + lane / LPR, c8 = 8 * (lane % LPR);
            if (!EVEN && (lane >= RPI * LPR || row >= 32)) continue;
            const int mo = m_wave + 32 * i + row, n = n_wave + c8;
            const uint4 q = *(const uint4 *)(strip + row * PITCH + c8);
            uint16_t *dst = g.out + (int64_t)mo * g.ldo + n;
            if (full) {
                typedef unsigned v4u __attribute__((ext_vector_type(4)));
                const v4u qv = {q.x, q.y, q.z, q.w};
                __builtin_nontemporal_store(qv, (v4u *)dst);  // streamed once, never re-read here
            } else if (mo < g.M && n < g.N) {
                const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (n + e < g.N) dst[e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
            }
        }
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    }
}

}  // namespace
}  // namespace bwta
