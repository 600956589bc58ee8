// Decode-shaped BWTA product on the FP4 matrix cores (up to 16 tokens against a large weight
// matrix).  The popcount decode kernel pays two vector-ALU operations per weight word PER TOKEN and
// a cross-lane reduction per output; here a weight word costs 7 vector-ALU operations whatever the
// token count and the reduction over k happens inside v_mfma_f32_16x16x128_f8f6f4, so the kernel
// stays bandwidth-bound up to the 16 tokens one instruction takes.
//
// Work split.  A workgroup owns T consecutive tiles of 16 output channels and all of K; K is cut
// into chunks of 512 (16 plane words) and wavefront w owns chunks [w RPW, (w+1) RPW).  Lane
// (i = lane % 16, g = lane / 16) of the instruction's first operand holds 32 k-values of channel i,
// of the second operand 32 k-values of token i; k-group g of chunk c is the 16 bytes at word
// 16 c + 4 g of the packed row and its four words feed the four instructions of the chunk.
// Because a dot product does not change when the same permutation of k is applied to both
// operands, bit 4 n + d of a word may go to nibble n of dword d in both operands, which is the
// cheapest expansion (shift, and-or).
//
//   weights: a wavefront streams its own 16 rows x RPW x 64 bytes of every tile with nontemporal
//            128-bit loads laid out along the rows (8 or more lanes per row: a direct
//            operand-order load would touch 16 different rows per 16 lanes) into a register ring
//            PF tiles deep, and turns them into operand order through a wavefront-private LDS
//            patch with an odd 16-byte pitch.  No workgroup barrier in the main loop.
//   tokens:  the wavefront's k-range of the mask/sign planes -> E2M1 nibbles in registers, once
//            per workgroup, reused for every tile
//   reduce:  every wavefront keeps a 16 x 16 fp32 partial per tile in registers; at the end the
//            workgroup sums them through LDS (exact: integers far below 2^24) and applies the
//            fused per-token x per-channel scale with a single rounding to fp16.
//
// One launch can walk several problems of the same shape (grid.y).
#include "bwta_internal.h"

namespace bwta {

namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));

struct DecodeBatch {
    static constexpr int MAX = 64;
    const uint32_t *mask[MAX], *sign[MAX], *wsign[MAX];
    const uint16_t *s_a[MAX], *s_w[MAX];
    int32_t *acc[MAX];
    uint16_t *out[MAX];
};

struct DecodeShape {
    int M, N, rw, a_mode, w_mode;  // M tokens in all; grid.z walks them in groups of 16
    int P;  // 16-byte pieces per packed row (rw / 4)
    int64_t ldo;
};

template <int RPW, int T, int PF, int MAXW>
__global__ __launch_bounds__(64 * MAXW) void k_gemv_fp4(DecodeBatch b, DecodeShape sh)
{
    constexpr int PW = 4 * RPW;          // pieces (16 bytes) per row in one wavefront's k-range
    constexpr int PITCH = PW + 1;        // LDS patch pitch in pieces (odd: conflict-free both ways)
    constexpr int TRMAX = MAXW > 8 ? 2 : 4;
    constexpr int TR = T < TRMAX ? T : TRMAX;  // tiles per reduction round (at most 32 KiB of partials)
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, KW = blockDim.x >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int p = blockIdx.y;
    const int tok0 = 16 * blockIdx.z;                                 // first token of this group
    const int Mg = sh.M - tok0 < 16 ? sh.M - tok0 : 16;               // tokens in it
    const int rw = sh.rw, P = sh.P;
    const int64_t tile0 = (int64_t)blockIdx.x * T;
    const uint32_t *wsign = b.wsign[p];
    extern __shared__ __attribute__((aligned(16))) v4u s_lds[];
    v4u *patch = s_lds + w * (16 * PITCH);              // this wavefront's transposition patch
    v4f *s_red = (v4f *)s_lds;                          // [TR][KW][64 lanes], reuses the patches at the end

    uint32_t m88 = 0x88888888u, c22 = 0x22222222u;  // kept opaque so each expansion is one v_and_or_b32
    asm volatile("" : "+s"(m88));
    asm volatile("" : "+v"(c22));

    // operand piece of this lane in chunk r: column PW w + 4 r + g of the row.  Past the row end the
    // token operand is zero, so whatever the weight operand holds there adds nothing.
    uint4 m4[RPW], s4[RPW];
    {
        const uint32_t *mask = b.mask[p] + (int64_t)tok0 * rw, *sign = b.sign[p] + (int64_t)tok0 * rw;
        const int tk = i < Mg ? i : 0;
#pragma unroll
        for (int r = 0; r < RPW; ++r) {
            const int c = PW * w + 4 * r + g;
            const bool live = c < P && i < Mg;
            const int cc = c < P ? c : 0;
            m4[r] = *(const uint4 *)(mask + (int64_t)tk * rw + 4 * cc);
            s4[r] = *(const uint4 *)(sign + (int64_t)tk * rw + 4 * cc);
            if (!live) m4[r] = make_uint4(0, 0, 0, 0);
        }
    }

    // streaming layout: piece q = lane + 64 j of the wavefront's 16 x PW patch -> row q / PW,
    // column q % PW.  Columns past the row end re-read column 0, rows past N the last row.
    // Addresses advance by a constant 16 rows per tile, so no multiplication in the loop.
    int srow[RPW], sdst[RPW];
    const v4u *sptr[RPW], *slast[RPW];  // piece of this lane in tile 0 / in the last row of the matrix
    const int row_first = 16 * (int)tile0;  // 16 * tiles < 2^31 + 16 T is guaranteed by the host
#pragma unroll
    for (int j = 0; j < RPW; ++j) {
        const int q = lane + 64 * j;
        srow[j] = q / PW;
        const int pc = q % PW, c = PW * w + pc;
        const int cc = c < P ? c : 0;
        sdst[j] = srow[j] * PITCH + pc;
        sptr[j] = (const v4u *)(wsign + (int64_t)(row_first + srow[j]) * rw) + cc;
        slast[j] = (const v4u *)(wsign + (int64_t)(sh.N - 1) * rw) + cc;
    }
    const int64_t tile_stride = 4 * (int64_t)rw;  // pieces per 16 rows
    // Rows that are whole 128-byte lines are streamed past the caches; otherwise neighbouring
    // wavefronts share the lines at the ends of their ranges, and a nontemporal load would fetch
    // those twice (measured: +22 % fetched bytes at K = 11008).
    const bool row_lines = (rw & 31) == 0;
    int next_row = row_first;
    auto load_next_tile = [&](v4u(&dst)[RPW]) {  // tiles are requested in order
#pragma unroll
        for (int j = 0; j < RPW; ++j) {
            const bool inside = next_row + srow[j] < sh.N;
            const v4u *src = inside ? sptr[j] : slast[j];
            dst[j] = row_lines ? __builtin_nontemporal_load(src) : *src;
            sptr[j] += tile_stride;
        }
        next_row += 16;
    };
    v4u ring[PF][RPW];
#pragma unroll
    for (int f = 0; f < PF; ++f)
        if (f < T) load_next_tile(ring[f]);

    // token operand (lane (i, g) = token i, k-group g), converted while the weights are in flight
    v8i tok[RPW][4];
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        const uint32_t mm[4] = {m4[r].x, m4[r].y, m4[r].z, m4[r].w};
        const uint32_t ss[4] = {s4[r].x & m4[r].x, s4[r].y & m4[r].y, s4[r].z & m4[r].z, s4[r].w & m4[r].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            v8i f;
            f[0] = (int)(((ss[e] << 3) & m88) | ((mm[e] << 1) & c22));
            f[1] = (int)(((ss[e] << 2) & m88) | (mm[e] & c22));
            f[2] = (int)(((ss[e] << 1) & m88) | ((mm[e] >> 1) & c22));
            f[3] = (int)((ss[e] & m88) | ((mm[e] >> 2) & c22));
            f[4] = f[5] = f[6] = f[7] = 0;
            tok[r][e] = f;
        }
    }

    v4f acc[T];
#pragma unroll
    for (int t = 0; t < T; ++t) {
        constexpr int dummy = 0;
        (void)dummy;
        const int f = t % PF;
#pragma unroll
        for (int j = 0; j < RPW; ++j) patch[sdst[j]] = ring[f][j];
        if (t + PF < T) load_next_tile(ring[f]);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        v4u x4[RPW];
#pragma unroll
        for (int r = 0; r < RPW; ++r) x4[r] = patch[i * PITCH + 4 * r + g];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        v4f a4 = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int r = 0; r < RPW; ++r)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t x = x4[r][e];
                v8i a;
                a[0] = (int)(((x << 3) & m88) | c22);
                a[1] = (int)(((x << 2) & m88) | c22);
                a[2] = (int)(((x << 1) & m88) | c22);
                a[3] = (int)((x & m88) | c22);
                a[4] = a[5] = a[6] = a[7] = 0;
                a4 = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, tok[r][e], a4, 4, 4, 0, 0, 0, 0);
            }
        acc[t] = a4;
    }

    // reduction over the wavefronts and epilogue, TR tiles per round.  Item x of a tile sums the KW
    // partials of token x / 4, channels 4 (x % 4) .. + 3  (accumulator layout: lane l, register v
    // -> channel 4 (l / 16) + v, token l % 16).
    const ScaleArg sa{b.s_a[p] && sh.a_mode == 2 ? b.s_a[p] + tok0 : b.s_a[p], b.s_a[p] ? sh.a_mode : 0};
    const ScaleArg sw{b.s_w[p], b.s_w[p] ? sh.w_mode : 0};
    int32_t *accp = b.acc[p] ? b.acc[p] + (int64_t)tok0 * sh.N : nullptr;
    uint16_t *out = b.out[p] ? b.out[p] + (int64_t)tok0 * sh.ldo : nullptr;
    const bool vec_ok = ((sh.ldo & 3) == 0) && (((uintptr_t)out & 7) == 0);
#pragma unroll
    for (int t0 = 0; t0 < T; t0 += TR) {
        __syncthreads();  // patches (first round) or the previous round's partials are no longer read
#pragma unroll
        for (int tt = 0; tt < TR; ++tt) s_red[(tt * KW + w) * 64 + lane] = acc[t0 + tt];
        __syncthreads();
        for (int idx = threadIdx.x; idx < TR * 64; idx += blockDim.x) {
            const int tt = idx >> 6, token = (idx & 63) >> 2, cg = idx & 3;
            v4f s = v4f{0.f, 0.f, 0.f, 0.f};
            for (int ww = 0; ww < KW; ++ww) s += s_red[(tt * KW + ww) * 64 + cg * 16 + token];
            const int64_t n = 16 * (tile0 + t0 + tt) + 4 * cg;
            if (token >= Mg || n >= sh.N) continue;
            const float fa = load_scale(sa, token);
            uint16_t *dstp = out + (int64_t)token * sh.ldo + n;
            int32_t *accq = accp + (int64_t)token * sh.N + n;
            if (n + 4 <= sh.N) {  // whole item inside the matrix: no per-element checks
                if (accp) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) accq[v] = (int)s[v];
                }
                if (out) {
                    float fw[4];
#pragma unroll
                    for (int v = 0; v < 4; ++v) fw[v] = fa * load_scale(sw, (int)n + v);
                    uint2 o;
                    o.x = scaled_to_half2(s[0], fw[0], s[1], fw[1]);
                    o.y = scaled_to_half2(s[2], fw[2], s[3], fw[3]);
                    if (vec_ok) {
                        *(uint2 *)dstp = o;
                    } else {
                        dstp[0] = (uint16_t)o.x, dstp[1] = (uint16_t)(o.x >> 16);
                        dstp[2] = (uint16_t)o.y, dstp[3] = (uint16_t)(o.y >> 16);
                    }
                }
            } else {
                for (int v = 0; v < 4 && n + v < sh.N; ++v) {
                    if (accp) accq[v] = (int)s[v];
                    if (out) dstp[v] = scaled_to_half(s[v], fa * load_scale(sw, (int)n + v));
                }
            }
        }
    }
}

int g_force_rpw = 0, g_force_t = 0, g_force_pf = 0;  // tuning override

template <int RPW, int T, int PF>
hipError_t launch_cfg(const DecodeBatch &b, int count, const DecodeShape &sh, hipStream_t st)
{
    const int KW = (sh.P + 4 * RPW - 1) / (4 * RPW);
    if (KW < 1 || KW > 16) return hipErrorInvalidValue;
    const int tiles = (sh.N + 15) / 16;
    const unsigned grid = (unsigned)((tiles + T - 1) / T);
    const int TR = T < (KW > 8 ? 2 : 4) ? T : (KW > 8 ? 2 : 4);
    const size_t lds_patch = (size_t)KW * 16 * (4 * RPW + 1) * 16, lds_red = (size_t)TR * KW * 1024;
    const size_t lds = lds_patch > lds_red ? lds_patch : lds_red;
    if (lds > 64 * 1024) return hipErrorInvalidValue;
    if (KW <= 4)
        hipLaunchKernelGGL((k_gemv_fp4<RPW, T, PF, 4>), dim3(grid, count, (sh.M + 15) / 16), dim3(64 * KW), lds, st, b, sh);
    else if (KW <= 8)
        hipLaunchKernelGGL((k_gemv_fp4<RPW, T, PF, 8>), dim3(grid, count, (sh.M + 15) / 16), dim3(64 * KW), lds, st, b, sh);
    else
        hipLaunchKernelGGL((k_gemv_fp4<RPW, T, PF, 16>), dim3(grid, count, (sh.M + 15) / 16), dim3(64 * KW), lds, st, b, sh);
    return hipGetLastError();
}

hipError_t launch_shape(const DecodeBatch &b, int count, const DecodeShape &sh, hipStream_t st)
{
    const int chunks = (sh.P + 3) / 4;
    const int tiles = (sh.N + 15) / 16;
    // chunks per wavefront: the smallest of 2..4 that needs at most 8 wavefronts, else at most 16
    int RPW = 2;
    while (RPW < 4 && (chunks + RPW - 1) / RPW > 8) ++RPW;
    if ((chunks + RPW - 1) / RPW > 8 && (chunks + 1) / 2 <= 16) RPW = 2;
    // tiles per workgroup: as many as still leave about 1024 workgroups in the launch
    const int64_t work = (int64_t)tiles * count * ((sh.M + 15) / 16);
    int T = work >= 8 * 1024 ? 8 : work >= 4 * 1024 ? 4 : 2;
    if (RPW >= 3 && T > 4) T = 4;
    int PF = T >= 4 ? 4 : 2;
    if (g_force_rpw) {
        if ((chunks + g_force_rpw - 1) / g_force_rpw <= 16) RPW = g_force_rpw;
        if (g_force_t) T = g_force_t;
        if (g_force_pf) PF = g_force_pf;
    }
#define BWTA_DEC(R_, T_, P_) if (RPW == R_ && T == T_ && PF == P_) return launch_cfg<R_, T_, P_>(b, count, sh, st);
    BWTA_DEC(1, 2, 2) BWTA_DEC(1, 8, 2) BWTA_DEC(1, 8, 4)
    BWTA_DEC(2, 2, 2) BWTA_DEC(2, 4, 2) BWTA_DEC(2, 8, 2) BWTA_DEC(2, 8, 4) BWTA_DEC(2, 16, 4)
    BWTA_DEC(3, 2, 2) BWTA_DEC(3, 4, 2) BWTA_DEC(3, 8, 2) BWTA_DEC(3, 8, 4) BWTA_DEC(3, 4, 4) BWTA_DEC(2, 4, 4) BWTA_DEC(4, 4, 4)
    BWTA_DEC(4, 2, 2) BWTA_DEC(4, 4, 2) BWTA_DEC(4, 8, 2) BWTA_DEC(4, 8, 4)
#undef BWTA_DEC
    return hipErrorInvalidValue;
}

}  // namespace

// 1..64 tokens (groups of 16 on grid.z, each streaming the weights: the repeats hit the caches);
// K up to 15 wavefronts x 4 chunks x 512 (their LDS patches fill 64 KiB)
bool gemv_fp4_supported(const GemmArgs &g)
{
    return g.M >= 1 && g.M <= 64 && g.N >= 1 && g.N <= (1 << 30) && g.rw >= 4 && (g.rw + 15) / 16 <= 60;
}

hipError_t launch_gemv_fp4_grouped(const GemmArgs *gs, int count, hipStream_t st)
{
    const GemmArgs &g0 = gs[0];
    for (int base = 0; base < count; base += DecodeBatch::MAX) {
        const int n = count - base < DecodeBatch::MAX ? count - base : DecodeBatch::MAX;
        DecodeBatch b;
        for (int i = 0; i < n; ++i) {
            const GemmArgs &g = gs[base + i];
            b.mask[i] = g.mask;
            b.sign[i] = g.sign;
            b.wsign[i] = g.wsign;
            b.s_a[i] = g.s_a.mode ? g.s_a.ptr : nullptr;
            b.s_w[i] = g.s_w.mode ? g.s_w.ptr : nullptr;
            b.acc[i] = g.acc;
            b.out[i] = g.out;
        }
        const int P = g0.rw / 4;
        DecodeShape sh{g0.M, g0.N, g0.rw, g0.s_a.mode, g0.s_w.mode, P, g0.ldo};
        hipError_t e = launch_shape(b, n, sh, st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_gemv_fp4(const GemmArgs &g, hipStream_t st) { return launch_gemv_fp4_grouped(&g, 1, st); }

void set_gemv_fp4_tile(int rpw, int t, int pf)
{
    g_force_rpw = rpw;
    g_force_t = t;
    g_force_pf = (pf == 2 || pf == 4) ? pf : 0;
}

}  // namespace bwta
