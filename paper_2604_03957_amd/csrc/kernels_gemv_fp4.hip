// Decode-shaped BWTA product on the FP4 matrix cores (up to 16 tokens per token group against a
// large weight matrix).  The popcount decode kernel pays two vector-ALU operations per weight word
// PER TOKEN and a cross-lane reduction per output; here a weight word costs 7 vector-ALU operations
// whatever the token count and the reduction over k happens inside v_mfma_f32_16x16x128_f8f6f4, so
// the kernel stays bandwidth-bound up to the 16 tokens one instruction takes.
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
//   weights: a wavefront streams its own 16 rows x RPW x 64 bytes of every tile with 128-bit
//            buffer loads laid out along the rows (8 or more lanes per row: a direct
//            operand-order load would touch 16 different rows per 16 lanes) into a register ring
//            PF tiles deep, and turns them into operand order through a wavefront-private LDS
//            patch with an odd 16-byte pitch.  The buffer descriptor ends at the workgroup's last
//            row, so the ring keeps issuing the same loads on every iteration (the hardware
//            answers the ones past the end with zeros and no memory traffic) and rows past N need
//            no address clamps.  No workgroup barrier in the main loop.
//   tokens:  the wavefront's k-range of the mask/sign planes -> E2M1 nibbles in registers, once
//            per workgroup, reused for every tile
//   reduce:  a wavefront's 16 x 16 partial of a tile is an integer of magnitude <= 512 RPW <= 2048,
//            exactly representable in fp16: it is parked in LDS as four halfs per lane right after
//            the tile (no accumulator registers held across tiles); after one barrier the
//            workgroup sums the partials in fp32 (exact) and applies the fused per-token x
//            per-channel scale with a single rounding to fp16.
//
// One launch can walk several problems of the same shape (grid.y).
//
// Measured and dropped: moving constant factors to the token operand (weight bits left in place as
// the E2M1 codes 0.5, 1, 2 and a sign; tokens carrying -4 t, -2 t, -t, +t; a per-token correction
// starting the accumulators) cuts the expansion from 7 to 4 operations per word and is exact, but
// the kernel is not bound by the vector ALU: no faster, and the extra registers cost occupancy.
#include <atomic>

#include "bwta_internal.h"

namespace bwta {

namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef __fp16 v2h __attribute__((ext_vector_type(2)));

struct DecodeBatch {
    static constexpr int MAX = 64;
    const uint32_t *mask[MAX], *sign[MAX], *wsign[MAX];
    const uint16_t *s_a[MAX], *s_w[MAX];
    int32_t *acc[MAX];
    uint16_t *out[MAX];
};

struct DecodeShape {
    int M, N, rw, a_mode, w_mode;  // M tokens in all, worked on in groups of 16
    int P;  // 16-byte pieces per packed row (rw / 4)
    int T;  // channel tiles per workgroup (a multiple of the ring depth)
    int G;  // token groups of 16 (ceil(M / 16)); NB = workgroups along the channels per group
    int64_t ldo;
};

union PartialBits {
    v2h h;
    uint32_t u;
};

template <int RPW, int PF, int MAXW, bool NT>
__global__ __launch_bounds__(64 * MAXW, MAXW == 4 && RPW <= 2 ? 5 : 4) void k_gemv_fp4(DecodeBatch b, DecodeShape sh)
{
    constexpr int PW = 4 * RPW;          // pieces (16 bytes) per row in one wavefront's k-range
    constexpr int PITCH = PW + 1;        // LDS patch pitch in pieces (odd: conflict-free both ways)
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, KW = blockDim.x >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int p = blockIdx.y;
    // Workgroups that stream the same weight rows for different token groups sit on the same XCD
    // (the hardware deals consecutive workgroup ids to the 8 XCDs in turn) and next to each other in
    // launch order, so the groups after the first find the rows in that XCD's L2:
    // id = 8 ((tb / 8) G + group) + tb % 8 for tile block tb.
    const int xq = blockIdx.x >> 3, tgroup = xq % sh.G;
    const int tblock = (xq / sh.G) * 8 + (blockIdx.x & 7);
    const int tok0 = 16 * tgroup;                                     // first token of this group
    const int Mg = sh.M - tok0 < 16 ? sh.M - tok0 : 16;               // tokens in it
    const int rw = sh.rw, P = sh.P, T = sh.T;
    const int64_t tile0 = (int64_t)tblock * T;
    if (16 * tile0 >= sh.N) return;  // the grid is padded to whole rounds of 8 tile blocks
    extern __shared__ __attribute__((aligned(16))) v4u s_lds[];
    v4u *patch = s_lds + w * (16 * PITCH);              // this wavefront's transposition patch
    uint2 *s_part = (uint2 *)(s_lds + KW * (16 * PITCH));  // [T][KW][64 lanes] x four halfs
    float *s_scale = (float *)(s_part + T * KW * 64);       // [16 T] channel scales, then [16] token scales

    // The scales the epilogue needs are requested before anything else and parked in LDS, so the
    // end of the workgroup waits on no global load.  Entry e < 16 T: channel 16 tile0 + e; then
    // 16 tokens.  The host keeps 16 T + 16 <= 2 blockDim.
    const ScaleArg sa{b.s_a[p] && sh.a_mode == 2 ? b.s_a[p] + tok0 : b.s_a[p], b.s_a[p] ? sh.a_mode : 0};
    const ScaleArg sw{b.s_w[p], b.s_w[p] ? sh.w_mode : 0};
    uint16_t my_scale[2];  // fp16 bits
    bool have_scale[2];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int e = threadIdx.x + k * blockDim.x;
        const int64_t n = 16 * tile0 + e;
        const bool chan = e < 16 * T;
        const bool use_w = chan && n < sh.N && sw.mode != 0;
        const bool use_a = !chan && e - 16 * T < Mg && sa.mode != 0;
        // every lane loads (an entry with no scale reads the matrix's first bytes and drops them),
        // so the request is issued here and first waited for where the value is parked
        const uint16_t *src = (const uint16_t *)b.wsign[p];
        if (use_w) src = sw.ptr + (sw.mode == 1 ? 0 : n);
        if (use_a) src = sa.ptr + (sa.mode == 1 ? 0 : e - 16 * T);
        have_scale[k] = use_w || use_a;
        my_scale[k] = *src;
    }

    uint32_t m88 = 0x88888888u, c22 = 0x22222222u;  // kept opaque so each expansion is one v_and_or_b32
    asm volatile("" : "+s"(m88));
    asm volatile("" : "+v"(c22));

    // streaming layout: piece q = lane + 64 j of the wavefront's 16 x PW patch -> row q / PW,
    // column q % PW (columns past the row end re-read column 0).  Byte offsets into the matrix fit
    // 32 bits (checked by the host) and advance by a constant 16 rows per tile; the descriptor's
    // size is the end of this workgroup's rows, clipped to the matrix.
    const int row_first = 16 * (int)tile0;
    const int row_end = row_first + 16 * T < sh.N ? row_first + 16 * T : sh.N;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void *)b.wsign[p], 0, (int)((uint32_t)row_end * (uint32_t)rw * 4u), 0x00020000);
    uint32_t voff[RPW], toff[RPW];
    int sdst[RPW];
#pragma unroll
    for (int j = 0; j < RPW; ++j) {
        const int q = lane + 64 * j;
        const int srow = q / PW, pc = q % PW, c = PW * w + pc;
        const int cc = c < P ? c : 0;
        sdst[j] = srow * PITCH + pc;
        toff[j] = ((uint32_t)srow * (uint32_t)rw + 4u * cc) * 4u;
        voff[j] = toff[j] + (uint32_t)row_first * (uint32_t)rw * 4u;
    }

    // The token planes of this group are fetched like one more tile (rows = tokens, so a request
    // covers whole row segments instead of 16 different rows per 16 lanes) and go through the same
    // patch into operand order.  Their descriptors end after token Mg - 1: further rows read zero,
    // and a zero mask is a zero token.
    v4u tm[RPW], ts[RPW];
    {
        const uint32_t tok_bytes = (uint32_t)Mg * (uint32_t)rw * 4u;
        const __amdgpu_buffer_rsrc_t rm = __builtin_amdgcn_make_buffer_rsrc(
            (void *)(b.mask[p] + (int64_t)tok0 * rw), 0, (int)tok_bytes, 0x00020000);
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
            (void *)(b.sign[p] + (int64_t)tok0 * rw), 0, (int)tok_bytes, 0x00020000);
#pragma unroll
        for (int j = 0; j < RPW; ++j) {
            tm[j] = __builtin_amdgcn_raw_buffer_load_b128(rm, (int)toff[j], 0, 0);
            ts[j] = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)toff[j], 0, 0);
        }
    }
    const uint32_t tile_bytes = 64u * (uint32_t)rw;  // 16 rows
    // Rows that are whole 128-byte lines are streamed past the caches; otherwise neighbouring
    // wavefronts share the lines at the ends of their ranges, and a nontemporal load would fetch
    // those twice (measured: +22 % fetched bytes at K = 11008).
    auto load_next_tile = [&](v4u(&dst)[RPW]) {  // tiles are requested in order
#pragma unroll
        for (int j = 0; j < RPW; ++j) {
            dst[j] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)voff[j], 0, NT ? 2 : 0);
            voff[j] += tile_bytes;
        }
    };
    v4u ring[PF][RPW];
#pragma unroll
    for (int f = 0; f < PF; ++f) {
        load_next_tile(ring[f]);
        __builtin_amdgcn_sched_barrier(0);  // keep the request order: the loop waits for the oldest tile only
    }

    // token operand (lane (i, g) = token i, k-group g): piece PW w + 4 r + g of the token's row.
    // Past the row end it is forced to zero, so whatever the weight operand holds there adds nothing.
    v4u m4[RPW], s4[RPW];
#pragma unroll
    for (int j = 0; j < RPW; ++j) patch[sdst[j]] = tm[j];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int r = 0; r < RPW; ++r) m4[r] = patch[i * PITCH + 4 * r + g];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int j = 0; j < RPW; ++j) patch[sdst[j]] = ts[j];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int r = 0; r < RPW; ++r) s4[r] = patch[i * PITCH + 4 * r + g];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    v8i tok[RPW][4];
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        const uint32_t keep = PW * w + 4 * r + g < P ? 0xffffffffu : 0u;
        const uint32_t mm[4] = {m4[r][0] & keep, m4[r][1] & keep, m4[r][2] & keep, m4[r][3] & keep};
        const uint32_t ss[4] = {s4[r][0] & mm[0], s4[r][1] & mm[1], s4[r][2] & mm[2], s4[r][3] & mm[3]};
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

    __builtin_amdgcn_sched_barrier(0);  // the scale requests are not waited for before this point
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int e = threadIdx.x + k * blockDim.x;
        if (e < 16 * T + 16) s_scale[e] = have_scale[k] ? half_bits_to_float(my_scale[k]) : 1.0f;
    }

    for (int t0 = 0; t0 < T; t0 += PF) {
#pragma unroll
        for (int f = 0; f < PF; ++f) {
#pragma unroll
            for (int j = 0; j < RPW; ++j) patch[sdst[j]] = ring[f][j];
            load_next_tile(ring[f]);  // tile t0 + f + PF; past the workgroup's last row it costs nothing
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
            PartialBits lo, hi;
            lo.h = __builtin_amdgcn_cvt_pkrtz(a4[0], a4[1]);  // exact: integers of magnitude <= 2048
            hi.h = __builtin_amdgcn_cvt_pkrtz(a4[2], a4[3]);
            s_part[((t0 + f) * KW + w) * 64 + lane] = make_uint2(lo.u, hi.u);
        }
    }

    // reduction over the wavefronts and epilogue.  Item x of a tile sums the KW partials of token
    // x / 4, channels 4 (x % 4) .. + 3  (accumulator layout: lane l, register v -> channel
    // 4 (l / 16) + v, token l % 16).
    int32_t *accp = b.acc[p] ? b.acc[p] + (int64_t)tok0 * sh.N : nullptr;
    uint16_t *out = b.out[p] ? b.out[p] + (int64_t)tok0 * sh.ldo : nullptr;
    const bool vec_ok = ((sh.ldo & 3) == 0) && (((uintptr_t)out & 7) == 0);
    __syncthreads();
    for (int idx = threadIdx.x; idx < T * 64; idx += blockDim.x) {
        const int tt = idx >> 6, token = (idx & 63) >> 2, cg = idx & 3;
        const int64_t n = 16 * (tile0 + tt) + 4 * cg;
        if (token >= Mg || n >= sh.N) continue;
        v4f s = v4f{0.f, 0.f, 0.f, 0.f};
        for (int ww = 0; ww < KW; ++ww) {
            const uint2 q = s_part[(tt * KW + ww) * 64 + cg * 16 + token];
            PartialBits lo, hi;
            lo.u = q.x;
            hi.u = q.y;
            s[0] += (float)lo.h[0];
            s[1] += (float)lo.h[1];
            s[2] += (float)hi.h[0];
            s[3] += (float)hi.h[1];
        }
        const float fa = s_scale[16 * T + token];
        const float *fwp = s_scale + 16 * tt + 4 * cg;
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
                for (int v = 0; v < 4; ++v) fw[v] = fa * fwp[v];
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
                if (out) dstp[v] = scaled_to_half(s[v], fa * fwp[v]);
            }
        }
    }
}

std::atomic<int> g_force_rpw{0}, g_force_t{0}, g_force_pf{0};  // tuning override (relaxed: a launch sees old or new)

size_t decode_lds_bytes(int RPW, int KW, int T)
{
    return (size_t)KW * 16 * (4 * RPW + 1) * 16 + (size_t)T * KW * 512 + (size_t)(16 * T + 16) * 4;
}

template <int RPW, int PF>
hipError_t launch_cfg(const DecodeBatch &b, int count, DecodeShape sh, hipStream_t st)
{
    const int KW = (sh.P + 4 * RPW - 1) / (4 * RPW);
    if (KW < 1 || KW > 16 || sh.T < PF || sh.T % PF != 0 || 16 * sh.T + 16 > 128 * KW) return hipErrorInvalidValue;
    const int tiles = (sh.N + 15) / 16;
    sh.G = (sh.M + 15) / 16;
    const int nb8 = ((tiles + sh.T - 1) / sh.T + 7) / 8 * 8;
    const dim3 grid((unsigned)(nb8 * sh.G), count, 1), block(64 * KW);
    const size_t lds = decode_lds_bytes(RPW, KW, sh.T);
    if (lds > 64 * 1024) return hipErrorInvalidValue;
    const bool nt = (sh.rw & 31) == 0 && sh.G == 1;  // later token groups are meant to hit the L2
#define BWTA_DEC_GO(MAXW_)                                                                      \
    do {                                                                                        \
        if (nt) hipLaunchKernelGGL((k_gemv_fp4<RPW, PF, MAXW_, true>), grid, block, lds, st, b, sh);  \
        else hipLaunchKernelGGL((k_gemv_fp4<RPW, PF, MAXW_, false>), grid, block, lds, st, b, sh);    \
    } while (0)
    if (KW <= 4) BWTA_DEC_GO(4);
    else if (KW <= 8) BWTA_DEC_GO(8);
    else BWTA_DEC_GO(16);
#undef BWTA_DEC_GO
    return hipGetLastError();
}

hipError_t launch_shape(const DecodeBatch &b, int count, DecodeShape sh, hipStream_t st)
{
    const int chunks = (sh.P + 3) / 4;
    const int tiles = (sh.N + 15) / 16;
    // chunks per wavefront: the smallest of 2..4 that needs at most 8 wavefronts, else at most 16
    int RPW = 2;
    while (RPW < 4 && (chunks + RPW - 1) / RPW > 8) ++RPW;
    if ((chunks + RPW - 1) / RPW > 8 && (chunks + 1) / 2 <= 16) RPW = 2;
    // tiles per workgroup: as many as still leave about 1024 workgroups in the launch
    const int64_t work = (int64_t)tiles * count * ((sh.M + 15) / 16);
    // (a single small matrix: one tile per workgroup, so that every compute unit gets one)
    int T = work >= 8 * 1024 ? 8 : work >= 4 * 1024 ? 4 : work >= 1024 ? 2 : 1;
    int PF = T == 1 ? 1 : RPW >= 3 ? 2 : T >= 4 ? 4 : 2;
    const int f_rpw = g_force_rpw.load(std::memory_order_relaxed), f_t = g_force_t.load(std::memory_order_relaxed),
              f_pf = g_force_pf.load(std::memory_order_relaxed);
    if (f_rpw) {
        if ((chunks + f_rpw - 1) / f_rpw <= 16) RPW = f_rpw;
        if (f_t) T = f_t;
        if (f_pf) PF = f_pf;
    }
    const int KW = (chunks + RPW - 1) / RPW;
    T = (T + PF - 1) / PF * PF;
    // partials must fit beside the patches, and two threads' worth of scale entries cover the tiles
    while (decode_lds_bytes(RPW, KW, T) > 64 * 1024 || 16 * T + 16 > 128 * KW) {
        if (T > PF) T -= PF;
        else if (PF > 2) PF = T = 2;
        else if (PF == 2) PF = T = 1;
        else break;
    }
    sh.T = T;
#define BWTA_DEC(R_, P_) if (RPW == R_ && PF == P_) return launch_cfg<R_, P_>(b, count, sh, st);
    BWTA_DEC(1, 1) BWTA_DEC(1, 2) BWTA_DEC(1, 3) BWTA_DEC(1, 4)
    BWTA_DEC(2, 1) BWTA_DEC(2, 2) BWTA_DEC(2, 3) BWTA_DEC(2, 4)
    BWTA_DEC(3, 1) BWTA_DEC(3, 2) BWTA_DEC(3, 3)
    BWTA_DEC(4, 1) BWTA_DEC(4, 2)  // deeper rings at 3 or 4 chunks per wavefront do not fit 128 registers
#undef BWTA_DEC
    return hipErrorInvalidValue;
}

}  // namespace

// 1..128 tokens (groups of 16 as neighbouring workgroups, each streaming the weights: the repeats hit L2;
// measured against the tiled kernel at 96 and 128 tokens: 5.9-13.5 us against 13.5-26 us on the 7B shapes);
// K up to 12 wavefronts x 4 chunks x 512 (their LDS patches and two tiles of partials fill 64 KiB)
bool gemv_fp4_supported(const GemmArgs &g)
{
    // byte offsets into a matrix, and a few workgroups' worth of rows past its end, must fit 32 bits
    const bool offsets_fit = ((int64_t)g.N + 4096) * g.rw * 4 <= 0xffffffffll;
    return g.M >= 1 && g.M <= 128 && g.N >= 1 && offsets_fit && g.rw >= 4 && (g.rw + 15) / 16 <= 48;
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
        // the call's scale modes: those of any problem that has the scale (one without reads as 1)
        int a_mode = 0, w_mode = 0;
        for (int i = 0; i < n; ++i) {
            if (gs[base + i].s_a.mode) a_mode = gs[base + i].s_a.mode;
            if (gs[base + i].s_w.mode) w_mode = gs[base + i].s_w.mode;
        }
        DecodeShape sh{g0.M, g0.N, g0.rw, a_mode, w_mode, P, 0, 1, g0.ldo};
        hipError_t e = launch_shape(b, n, sh, st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_gemv_fp4(const GemmArgs &g, hipStream_t st) { return launch_gemv_fp4_grouped(&g, 1, st); }

void set_gemv_fp4_tile(int rpw, int t, int pf)
{
    g_force_rpw.store(rpw, std::memory_order_relaxed);
    g_force_t.store(t, std::memory_order_relaxed);
    g_force_pf.store((pf >= 1 && pf <= 4) ? pf : 0, std::memory_order_relaxed);
}

}  // namespace bwta
