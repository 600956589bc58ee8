// BWTA product on the FP4 matrix cores (v_mfma_f32_32x32x64_f8f6f4, both operands E2M1).
//
// +1, -1 and 0 are exact E2M1 values (0b0010, 0b1010, 0b0000) and every partial sum is an
// integer below 2^24, so the fp32 accumulators hold the exact BWTA product (Case 1 of the
// paper's arithmetic rules) while the instruction retires twice the MACs of the int8 form.
//   * Activations are converted once per call from the two bit planes into E2M1 nibbles
//     (bit 1 = mask, bit 3 = sign) in a fragment-major layout: [row block of 32][k step of
//     64][lane][4 dwords].  A wavefront's operand for one instruction is one contiguous
//     kilobyte, which it loads straight from global memory (L2) into registers, eight k steps
//     ahead of use; activations never touch LDS.
//   * Weights stay one bit each in HBM and LDS; a lane widens the 32 bits it needs for one
//     instruction into four dwords of nibbles with three shifts and four and-or ops.
// The dot product does not depend on the order of k inside an instruction, so element
// 4 i + d of a 32-bit word goes to nibble i of dword d in BOTH operands, which is what makes
// the widening that cheap.
// The weights are the instruction's first operand, so a lane ends up with 4 consecutive output
// channels of one token: the fp16 epilogue packs them and moves 8 bytes per LDS write.
//
// Kernels here: k_planes_to_fp4 / k_quantize_to_fp4 (bit planes / fp16 activations -> fragments),
// k_gemm_fp4 (the tiled product) and k_linear_fused (ternarise + product in one launch, short K).
#include <atomic>
#include <type_traits>

#include "bwta_internal.h"
#include "bwta_fp4_tile.h"

namespace bwta {

namespace {

// planes -> E2M1 fragments.  A workgroup converts 32 rows x NW words: plane rows are read with
// coalesced 128-bit loads, the nibble dwords are regrouped through LDS, and the NW / 2 KiB of
// fragments it produces (NW / 2 k steps of one row block) leave as one contiguous run.  The buffer
// is padded with zeros to a multiple of 8 row blocks and 8 k steps so that the GEMM never has
// to guard an activation load.  The kernel is one memory round trip long, so small problems take
// small NW: more workgroups, and every compute unit has requests in flight from the start.
template <int NW>  // 8, 16 or 32 plane words per workgroup of 8 NW threads
__global__ __launch_bounds__(8 * NW) void k_planes_to_fp4(const uint32_t *__restrict__ mask,
                                                          const uint32_t *__restrict__ sign, int M, int K, int rw,
                                                          int s_pad, uint32_t *__restrict__ frag)
{
    __shared__ uint4 tile[NW * 33];  // [slot = step_local * 2 + half][row], one spare row of skew
    constexpr int NT = 8 * NW, QPR = NW / 4;  // threads; 128-bit pieces per row
    const int t = threadIdx.x;
    const int rb = blockIdx.y, wc = blockIdx.x;  // row block, group of NW words (NW / 2 k steps)
    const int row = t / QPR, q4 = t % QPR;
    const int m = rb * 32 + row, q = NW * wc + 4 * q4;
    uint4 mk4 = make_uint4(0, 0, 0, 0), sg4 = mk4;
    if (m < M && q < rw) {
        sg4 = *(const uint4 *)(sign + (int64_t)m * rw + q);
        if (mask) {
            mk4 = *(const uint4 *)(mask + (int64_t)m * rw + q);
        } else {  // binary (+-1) activations: every element below K is non-zero, no mask plane is read
            uint32_t ones[4];
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const int left = K - 32 * (q + w);
                ones[w] = left >= 32 ? 0xffffffffu : (left > 0 ? (1u << left) - 1u : 0u);
            }
            mk4 = make_uint4(ones[0], ones[1], ones[2], ones[3]);
        }
    }
    const uint32_t mks[4] = {mk4.x, mk4.y, mk4.z, mk4.w};
    const uint32_t sgs[4] = {sg4.x, sg4.y, sg4.z, sg4.w};
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const uint32_t mk = mks[w], sg = sgs[w] & mk;
        uint4 o;
        o.x = ((sg << 3) & 0x88888888u) | ((mk << 1) & 0x22222222u);
        o.y = ((sg << 2) & 0x88888888u) | (mk & 0x22222222u);
        o.z = ((sg << 1) & 0x88888888u) | ((mk >> 1) & 0x22222222u);
        o.w = (sg & 0x88888888u) | ((mk >> 2) & 0x22222222u);
        int step, half;
        word_slot(4 * q4 + w, step, half);  // local word index 0..NW-1 -> local step 0..NW/2-1
        tile[(step * 2 + half) * 33 + row] = o;
    }
    __syncthreads();
    uint4 *dst = (uint4 *)frag + ((int64_t)rb * s_pad + (NW / 2) * wc) * 64;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int idx = t + NT * k;  // 16-byte piece of the output run: slot idx/32, row idx%32
        if ((NW / 2) * wc + (idx >> 6) < s_pad) dst[idx] = tile[(idx >> 5) * 33 + (idx & 31)];
    }
}

// fp16 activations -> E2M1 fragments in one pass (ternarise by the paper's threshold rule and
// emit the GEMM operand directly; no bit planes in between).  A lane takes 8 consecutive
// elements (one 128-bit load); the 4 lanes of a quad cover one 32-element word, whose 4 nibble
// dwords are assembled with a byte transpose inside the quad.  Quads of a wavefront walk
// consecutive rows, so the 16-byte fragments they store are contiguous.
// QF_R: k steps (2 plane words) per thread; more than one amortises constants and addressing when
// the launch still has enough workgroups to fill the chip.
template <int QF_R>
__global__ __launch_bounds__(256) void k_quantize_to_fp4(const uint16_t *__restrict__ A, int64_t lda, ScaleArg s_a,
                                                         int M, int K, int s_pad, uint32_t *__restrict__ frag,
                                                         int vec_ok)
{
    const int t = threadIdx.x;
    const int quad = t >> 2, j = t & 3;
    const int row = quad & 31;  // row in block
    const int rb = blockIdx.y, m = rb * 32 + row;
    const int q0 = 2 * QF_R * blockIdx.x + (quad >> 5);  // first plane word of this quad; then every second one

    // The scale is requested first and every data load right behind it; nothing is waited for
    // until all of the thread's requests are out (a wait in front of the data loads would put one
    // memory round trip in front of the other in every workgroup).
    const int mc = m < M ? m : 0;
    const bool have_scale = s_a.mode != 0 && s_a.ptr != nullptr;
    const uint16_t s_bits = *(have_scale ? s_a.ptr + (s_a.mode == 1 ? 0 : mc) : A);  // no scale: a dropped read

    uint4 x[QF_R];
    if (vec_ok) {  // rows are 16-byte aligned and K is a multiple of 8: whole 128-bit loads only
#pragma unroll
        for (int it = 0; it < QF_R; ++it) {
            const int k0 = 32 * (q0 + 2 * it) + 8 * j;
            const bool inb = m < M && k0 < K;  // lanes outside re-read the first bytes and drop them
            x[it] = *(const uint4 *)(A + (inb ? (int64_t)m * lda + k0 : 0));
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int it = 0; it < QF_R; ++it) {
            const int k0 = 32 * (q0 + 2 * it) + 8 * j;
            if (!(m < M && k0 < K)) x[it] = make_uint4(0, 0, 0, 0);
        }
    } else {
#pragma unroll
        for (int it = 0; it < QF_R; ++it) {
            const int k0 = 32 * (q0 + 2 * it) + 8 * j;
            x[it] = make_uint4(0, 0, 0, 0);
            if (m < M && k0 < K) {
                const uint16_t *src = A + (int64_t)m * lda + k0;
                const int nvalid = K - k0 >= 8 ? 8 : K - k0;
                uint16_t v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = e < nvalid ? src[e] : (uint16_t)0;
                x[it] = make_uint4(v[0] | ((uint32_t)v[1] << 16), v[2] | ((uint32_t)v[3] << 16),
                                   v[4] | ((uint32_t)v[5] << 16), v[6] | ((uint32_t)v[7] << 16));
            }
        }
    }

    // An invalid scale (and a row past M) ternarises to zero; elements past K are loaded as +0 and
    // are zero under every valid threshold, so the element loop needs no validity logic.
    const TernaryThr thr = ternary_thresholds(have_scale ? s_bits : 0x3c00u, m < M);

#pragma unroll
    for (int it = 0; it < QF_R; ++it) {
        const int q = q0 + 2 * it;
        const uint32_t D = fragment_dword(x[it], thr, j);
        int step, half;
        word_slot(q, step, half);
        if (step < s_pad) frag[(((int64_t)rb * s_pad + step) * 64 + half * 32 + row) * 4 + j] = D;
    }
}

// bits of a boolean operand -> E2M1 nibbles (1 = 0b0010 = +1, 0 = 0b0000), same element order
__device__ __forceinline__ v8i widen_bool(uint32_t x, uint32_t c22)
{
    v8i r;
    r[0] = (int)((x << 1) & c22);
    r[1] = (int)(x & c22);
    r[2] = (int)((x >> 1) & c22);
    r[3] = (int)((x >> 2) & c22);
    r[4] = r[5] = r[6] = r[7] = 0;
    return r;
}

// MODE 1 of k_gemm_fp4 (the BWTA_Att product: boolean attention plane x prepared ternary V^T, one
// batch entry per blockIdx.y): where batch b's operands and output start, and the scale prefix
struct BatchArgs {
    int64_t frag_stride_dw, w_stride_words, out_stride;
    float alpha;
    int batch;
};

constexpr int WD_PITCH = 20;  // dwords per LDS weight row: 16 words (512 k) + 4 pad

// KS > 1: the K loop is split over KS groups of wavefronts inside the workgroup (each group owns
// every KS-th 512-k slab); their partial accumulators are summed through LDS before the epilogue.
// Used when a shape has too few output tiles to fill the chip.
template <int WM, int WN, int WAVES_M, int WAVES_N, int KS>
struct Cfg {
    static constexpr int BM = 32 * WM * WAVES_M, BN = 32 * WN * WAVES_N;
    static constexpr int GROUP_WAVES = WAVES_M * WAVES_N;
    static constexpr int THREADS = 64 * GROUP_WAVES * KS;
    static constexpr int W_DW = BN * WD_PITCH;           // one group's 512-k slab
    static constexpr int W_PIECES = BN * 4 * KS;         // 16-byte pieces per iteration
    static constexpr int W_LOADS = (W_PIECES + THREADS - 1) / THREADS;
    static constexpr int STRIP_HALFS = 32 * (32 * WN + 8);  // per wavefront: 32 tokens x 32*WN channels
    static constexpr int EPI_BYTES = BN * 4 + GROUP_WAVES * STRIP_HALFS * 2;
    static constexpr int RED_BYTES = KS > 1 ? GROUP_WAVES * WM * WN * 16 * 64 * 4 : 0;
    static constexpr int LOOP_BYTES = 2 * KS * W_DW * 4;
    static constexpr int WORK_BYTES =
        (LOOP_BYTES > EPI_BYTES ? LOOP_BYTES : EPI_BYTES) > RED_BYTES ? (LOOP_BYTES > EPI_BYTES ? LOOP_BYTES : EPI_BYTES)
                                                                      : RED_BYTES;
    static constexpr int SCALE_BYTES = (BN + BM) * 4;  // the tile's s_w and s_a as floats, fetched at the start
    static constexpr int SMEM_BYTES = WORK_BYTES + SCALE_BYTES;
    static_assert(BN <= THREADS && BM <= THREADS, "one thread per scale");
};

// MODE 0: the linear layer.  MODE 1: the BWTA_Att product of the attention block, batched over
// heads (a group of workgroups per head).  The 1-bit operand ("weights": N rows) is the boolean attention plane, whose
// set bits count +1 and clear bits 0; the fragment operand ("activations": M rows) is V^T prepared
// like an activation; the MFMA operands swap places, so a lane ends up with 4 consecutive rows of
// V^T (head-dimension entries) for one attention row and the epilogue writes out[n][m], the
// context matrix, with the scale fp32(alpha * (s_a * s_w)).
template <int WM, int WN, int WAVES_M, int WAVES_N, int OCC, bool WITH_ACC, int KS, int D, int MODE>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N * KS) __attribute__((amdgpu_waves_per_eu(OCC, OCC)))
void k_gemm_fp4(GemmArgs g, const uint32_t *__restrict__ frag, int s_pad, int tiles_n, int tiles_total, BatchArgs ba)
{
    using C = Cfg<WM, WN, WAVES_M, WAVES_N, KS>;
    static_assert(MODE == 0 || (WM == WN && KS == 1 && !WITH_ACC), "the swapped epilogue reuses the strips as they are");
    int tm, tn;
    if constexpr (MODE == 1) {
        // One batch entry (head) per group of tiles_total workgroups.  With a multiple of 8 entries
        // the groups are dealt to the XCDs whole (the hardware sends consecutive workgroup ids to the 8
        // XCDs in turn): all tiles of a head then share one L2, which fetches that head's V^T
        // fragments once instead of once per XCD.
        int64_t bz;
        if ((ba.batch & 7) == 0) {
            const int L = blockIdx.x, k = L >> 3;
            bz = (L & 7) + 8 * (k / tiles_total);
            const int t = k % tiles_total;
            tm = t % (tiles_total / tiles_n);
            tn = t / (tiles_total / tiles_n);
        } else {
            bz = blockIdx.x / tiles_total;
            const int t = blockIdx.x % tiles_total;
            tm = t % (tiles_total / tiles_n);
            tn = t / (tiles_total / tiles_n);
        }
        frag += bz * ba.frag_stride_dw;
        g.wsign += bz * ba.w_stride_words;
        g.out += bz * ba.out_stride;
        if (g.s_a.mode == 2 && g.s_a.ptr) g.s_a.ptr += bz * g.M;
        if (g.s_w.mode == 2 && g.s_w.ptr) g.s_w.ptr += bz * g.N;
    }
    static_assert(D == 8 || D == 16, "activation prefetch distance in k steps: one or two slabs");
    extern __shared__ __attribute__((aligned(16))) uint32_t smem[];

    if constexpr (MODE == 0) tile_of_workgroup(tiles_n, tiles_total, tm, tn);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int kg = KS == 1 ? 0 : wave / C::GROUP_WAVES;  // k group
    const int wl = KS == 1 ? wave : wave % C::GROUP_WAVES;  // wavefront within the group
    const int wm = wl / WAVES_N, wn = wl % WAVES_N;
    const int r32 = lane & 31, h = lane >> 5;
    const int m0 = tm * C::BM, n0 = tn * C::BN;
    const int rw = g.rw;
    const int npairs = s_pad / 8;  // slabs of 8 k steps (512 k); the fragment buffer is padded to that
    const int niter = (npairs + KS - 1) / KS;
    const int nsteps = rw >> 1;  // k steps of 64 that hold data (rw is a multiple of 4 words)

    uint32_t m88 = 0x88888888u, c22 = 0x22222222u;
    asm volatile("" : "+s"(m88));
    asm volatile("" : "+v"(c22));

    // this wavefront's activation fragments: row blocks rbw .. rbw+WM-1, one KiB per (block, step).
    // Loads are never predicated: steps past the end are clamped to the last step (the value is
    // loaded but never used).
    const uint4 *abase = (const uint4 *)frag + ((int64_t)(tm * (C::BM / 32) + wm * WM) * s_pad) * 64 + lane;
    const int last_step = s_pad - 1;
    auto load_a = [&](uint4 (&dst)[WM], int step) {
        const int st = step < last_step ? step : last_step;
#pragma unroll
        for (int i = 0; i < WM; ++i) dst[i] = abase[((int64_t)i * s_pad + st) * 64];
    };

    // weight words of 512 k; rows / words past the end are clamped (their products meet zero
    // activations or land in channels that are never stored)
    // Weight slabs are requested WPF iterations before they are staged: one iteration of 8 k steps
    // is shorter than a trip to memory when only one or two wavefronts share a SIMD.
    constexpr int WPF = OCC >= 3 ? 1 : 2;
    uint4 pwbuf[WPF][C::W_LOADS];
    auto fetch_w = [&](int it, uint4 (&pw)[C::W_LOADS]) {  // slabs it*KS .. it*KS+KS-1, one per k group
#pragma unroll
        for (int i = 0; i < C::W_LOADS; ++i) {
            const int p = tid + i * C::THREADS;  // piece: group p/(4 BN), row (p/4)%BN, quarter p%4
            int n = n0 + (KS == 1 ? (p >> 2) : ((p >> 2) % C::BN));
            int kw = 16 * (it * KS + (KS == 1 ? 0 : p / (4 * C::BN))) + 4 * (p & 3);
            n = n < g.N ? n : g.N - 1;
            kw = kw < rw ? kw : rw - 4;
            if (C::W_PIECES % C::THREADS == 0 || p < C::W_PIECES)
                pw[i] = *(const uint4 *)(g.wsign + (int64_t)n * rw + kw);
        }
    };
    auto stage_w = [&](int buf, const uint4 (&pw)[C::W_LOADS]) {
        uint32_t *sW = smem + buf * KS * C::W_DW;
#pragma unroll
        for (int i = 0; i < C::W_LOADS; ++i) {
            const int p = tid + i * C::THREADS;
            if (C::W_PIECES % C::THREADS == 0 || p < C::W_PIECES) {
                // each chunk's words w0..w7 are stored as [w0 w1 w4 w5 | w2 w3 w6 w7] so that lane
                // half h finds the words of its steps 0..3 in one 16-byte read at 4 h
                uint32_t *row = sW + (p >> 2) * WD_PITCH + 8 * ((p >> 1) & 1);  // (p>>2) = group * BN + row
                const int half = p & 1;
                *(uint2 *)(row + 2 * half) = make_uint2(pw[i].x, pw[i].y);
                *(uint2 *)(row + 4 + 2 * half) = make_uint2(pw[i].z, pw[i].w);
            }
        }
    };

    v16f acc[WN][WM];  // [channel block][token block]: rows of the MFMA result are channels
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
        for (int i = 0; i < WM; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][i][v] = 0.0f;

    // The tile's scales are requested before anything else and parked in LDS with the first weight
    // slab, so the epilogue never waits on a global load.
    float *sc_lds = (float *)(smem + C::WORK_BYTES / 4);  // [BN] channel scales, then [BM] token scales
    // Every thread issues both loads (one with nothing to fetch re-reads the weights' first bytes and
    // drops them) and the bits are converted only where they are parked: a conditional load is
    // waited for inside its branch, which would put two memory round trips in front of the
    // operand requests of every workgroup.
    const bool want_sw = tid < C::BN && n0 + tid < g.N, want_sa = tid < C::BM && m0 + tid < g.M;
    const bool have_sw = want_sw && g.s_w.mode != 0 && g.s_w.ptr != nullptr;
    const bool have_sa = want_sa && g.s_a.mode != 0 && g.s_a.ptr != nullptr;
    const uint16_t *scale_safe = (const uint16_t *)g.wsign;
    const uint16_t sw_bits = *(have_sw ? g.s_w.ptr + (g.s_w.mode == 1 ? 0 : n0 + tid) : scale_safe);
    const uint16_t sa_bits = *(have_sa ? g.s_a.ptr + (g.s_a.mode == 1 ? 0 : m0 + tid) : scale_safe);
    __builtin_amdgcn_sched_barrier(0);  // requested first, so parking them waits for nothing younger

    uint4 ring[D][WM];
    fetch_w(0, pwbuf[0]);
#pragma unroll
    for (int s = 0; s < D; ++s) load_a(ring[s], 8 * (kg + KS * (s / 8)) + (s & 7));
    stage_w(0, pwbuf[0]);
    if (WPF == 2 && niter > 1) fetch_w(1, pwbuf[WPF - 1]);  // staged at the end of iteration 0
    if (tid < C::BN) sc_lds[tid] = have_sw ? half_bits_to_float(sw_bits) : (want_sw ? 1.0f : 0.0f);
    if (tid < C::BM) sc_lds[C::BN + tid] = have_sa ? half_bits_to_float(sa_bits) : (want_sa ? 1.0f : 0.0f);
    __syncthreads();

    int buf = 0;
    // Every path through a full iteration issues the same loads (weight slab always, clamped to the
    // last one; ring refills always, clamped to the last step), so the wait counters the compiler
    // derives do not collapse to the shortest path.  A last slab that holds data only in its first
    // four steps (K = 768: 12 steps) runs as a peeled half iteration without any loads.
    auto iteration = [&](int it, auto parity, auto half_only) {
        constexpr int PAR = decltype(parity)::value;    // it & 1
        constexpr bool HALF = decltype(half_only)::value;
        constexpr int RH = D == 16 ? PAR : 0;           // which half of a 16-deep ring this slab uses
        constexpr int PWN = WPF == 2 ? PAR : 0;         // registers that receive the slab requested now
        constexpr int PWS = WPF == 2 ? PAR ^ 1 : 0;     // registers that hold the slab staged at the end
        const int pr = it * KS + kg;  // this group's slab
        const uint32_t *sW = smem + (buf * KS + kg) * C::W_DW;
        const bool more = it + 1 < niter;
        if (!HALF) fetch_w(it + WPF < niter ? it + WPF : niter - 1, pwbuf[PWN]);  // staging only waits for older loads
        uint4 xw[2][WN];
#pragma unroll
        for (int sub = 0; sub < (HALF ? 1 : 2); ++sub)
#pragma unroll
            for (int j = 0; j < WN; ++j)
                xw[sub][j] = *(const uint4 *)(sW + ((wn * WN + j) * 32 + r32) * WD_PITCH + 8 * sub + 4 * h);
        if (KS == 1 || pr < npairs) {
#pragma unroll
        for (int s8 = 0; s8 < (HALF ? 4 : 8); ++s8) {
            const int slot = (8 * RH + s8) % D, sub = s8 >> 2, s = s8 & 3;
            v8i a[WM], b[WN];
#pragma unroll
            for (int i = 0; i < WM; ++i) {
                a[i][0] = (int)ring[slot][i].x; a[i][1] = (int)ring[slot][i].y;
                a[i][2] = (int)ring[slot][i].z; a[i][3] = (int)ring[slot][i].w;
                a[i][4] = a[i][5] = a[i][6] = a[i][7] = 0;
            }
#pragma unroll
            for (int j = 0; j < WN; ++j) {
                const uint4 x = xw[sub][j];
                const uint32_t wbits = s == 0 ? x.x : s == 1 ? x.y : s == 2 ? x.z : x.w;
                if constexpr (MODE == 1) b[j] = widen_bool(wbits, c22);
                else b[j] = widen_w(wbits, m88, c22);
            }
#pragma unroll
            for (int j = 0; j < WN; ++j)
#pragma unroll
                for (int i = 0; i < WM; ++i)
                    if constexpr (MODE == 1)
                        acc[j][i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[i], b[j], acc[j][i], 4, 4, 0, 0, 0, 0);
                    else
                        acc[j][i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b[j], a[i], acc[j][i], 4, 4, 0, 0, 0, 0);
            if (!HALF) load_a(ring[slot], 8 * (pr + KS * (D / 8)) + s8);  // refill the slot D steps of this group ahead
        }
        }
        if (!HALF && more) stage_w(buf ^ 1, pwbuf[PWS]);  // nothing to stage after the last slab
        __syncthreads();
        buf ^= 1;
    };
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    const bool tail_half = KS == 1 && (nsteps & 7) != 0 && (nsteps & 7) <= 4;
    const int nfull = niter - (tail_half ? 1 : 0);
    if constexpr (WPF == 1 && D == 8) {  // nothing depends on the parity: one copy of the body
        for (int it = 0; it < nfull; ++it) iteration(it, P0{}, std::false_type{});
        if (tail_half) iteration(nfull, P0{}, std::true_type{});
    } else {
        for (int it = 0; it < nfull; it += 2) {
            iteration(it, P0{}, std::false_type{});
            if (it + 1 < nfull) iteration(it + 1, P1{}, std::false_type{});
        }
        if (tail_half) {
            if (nfull & 1)
                iteration(nfull, P1{}, std::true_type{});
            else
                iteration(nfull, P0{}, std::true_type{});
        }
    }

    // ---- sum the k groups' partial accumulators into group 0 (one group at a time through LDS)
    if (KS > 1) {
        float *red = (float *)smem;  // [wavefront in group][register][lane]; the weight slabs are dead
        for (int r = 1; r < KS; ++r) {
            if (kg == r) {
#pragma unroll
                for (int j = 0; j < WN; ++j)
#pragma unroll
                    for (int i = 0; i < WM; ++i)
#pragma unroll
                        for (int v = 0; v < 16; ++v)
                            red[((wl * WN * WM + j * WM + i) * 16 + v) * 64 + lane] = acc[j][i][v];
            }
            __syncthreads();
            if (kg == 0) {
#pragma unroll
                for (int j = 0; j < WN; ++j)
#pragma unroll
                    for (int i = 0; i < WM; ++i)
#pragma unroll
                        for (int v = 0; v < 16; ++v)
                            acc[j][i][v] += red[((wl * WN * WM + j * WM + i) * 16 + v) * 64 + lane];
            }
            __syncthreads();
        }
    }

    // ---- epilogue (k group 0 only).  Lane (r32, h) of block (j, i) holds token m = 32 i + r32 and
    // channels n = 32 j + 8 g + 4 h + q (register v = 4 g + q).
    const int m_wave = m0 + wm * WM * 32, n_wave = n0 + wn * WN * 32;
    if (WITH_ACC && g.acc && kg == 0) {
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            const int m = m_wave + 32 * i + r32;
#pragma unroll
            for (int j = 0; j < WN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int n = n_wave + 32 * j + 8 * (v >> 2) + 4 * h + (v & 3);
                    if (m < g.M && n < g.N) g.acc[(int64_t)m * g.N + n] = (int)acc[j][i][v];
                }
        }
    }
    if (!g.out) return;

    const float *sw_lds = sc_lds, *sa_lds = sc_lds + C::BN;
    // the loop's last barrier retired every read of the weight slabs, whose LDS the strips reuse
    uint16_t *strip = (uint16_t *)(smem + C::BN) + wl * C::STRIP_HALFS;
    if (kg != 0) return;  // no barrier below this point
    if constexpr (MODE == 1) {
        // lane (r32, h) of block (j, i) holds attention row 32 j + r32 and V^T rows 32 i + 8 g + 4 h + q:
        // the same epilogue with the two sides exchanged
        v16f acct[WM][WN];
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int i = 0; i < WM; ++i) acct[i][j] = acc[j][i];
        GemmArgs gs = g;
        gs.M = g.N;
        gs.N = g.M;
        store_tile_fp16<WN, WM, true>(acct, gs, sw_lds + wn * WN * 32, sa_lds + wm * WM * 32, strip, n_wave, m_wave, lane,
                                      ba.alpha);
    } else {
        store_tile_fp16<WM, WN>(acc, g, sa_lds + wm * WM * 32, sw_lds + wn * WN * 32, strip, m_wave, n_wave, lane);
    }
}

template <int WM, int WN, int WAVES_M, int WAVES_N, int OCC, bool WITH_ACC, int KS = 1, int D = 8, int MODE = 0>
hipError_t launch(const GemmArgs &g, const uint32_t *frag, int s_pad, hipStream_t st, int batch = 1,
                  BatchArgs ba = BatchArgs{0, 0, 0, 1.0f, 1})
{
    using C = Cfg<WM, WN, WAVES_M, WAVES_N, KS>;
    static bool configured = false;  // benign race: setting the attribute twice is harmless
    if (!configured) {
        hipError_t e = hipFuncSetAttribute((const void *)k_gemm_fp4<WM, WN, WAVES_M, WAVES_N, OCC, WITH_ACC, KS, D, MODE>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, C::SMEM_BYTES);
        if (e != hipSuccess) return e;
        configured = true;
    }
    const int tiles_n = (g.N + C::BN - 1) / C::BN, tiles_m = (g.M + C::BM - 1) / C::BM;
    const int64_t total = (int64_t)tiles_n * tiles_m;
    if (total > 0x7fffffff) return hipErrorInvalidValue;
    if (total * batch > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL((k_gemm_fp4<WM, WN, WAVES_M, WAVES_N, OCC, WITH_ACC, KS, D, MODE>), dim3((unsigned)(total * batch)),
                       dim3(C::THREADS), C::SMEM_BYTES, st, g, frag, s_pad, tiles_n, (int)total, ba);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// bwta_linear in one launch for short K (K <= 1024): ternarise + product + epilogue.  With fp16
// activations in and few k steps per output, the two-kernel form spends most of its time on what a
// launch costs however little it computes (ramp, one memory round trip before the first
// instruction that needs data, drain) and on writing and re-reading the fragments.
// A workgroup owns one strip of 32 tokens and 1/R of the channels.  It ternarises its strip straight
// into LDS in MFMA operand order (all of K: at most 16 KiB), so the activation operand of every
// MFMA comes from LDS and is shared by all channels; the R workgroups of a strip repeat that part.
// Each wavefront then walks its channel blocks two at a time: the weight bits of a group are
// loaded from global memory directly in operand layout (lane (r, h) takes four words of row r; the
// fragments are produced here, so words are dealt to k steps in the order that makes those four
// words adjacent), all of K at once, and requested a group ahead, so the K loop runs out of
// registers and LDS and the wavefronts share no barrier after the first: their epilogues and
// stores overlap the others' MFMAs.
constexpr int FL_STRIP_HALFS = 32 * (32 * 2 + 8);  // room for the widest group

// word j of a 256-k chunk feeds k step j % 4 of the chunk on lane half j / 4
template <int NCH, int FL_CB, int NWV>  // 256-k chunks of K (1..4); channel blocks (of 32) per group: 1 or 2; wavefronts: 4 or 8
__global__ __launch_bounds__(64 * NWV) void k_linear_fused(const uint16_t *__restrict__ A, int64_t lda, GemmArgs g, int R,
                                                      int cbw /* channel blocks per workgroup, a multiple of NWV FL_CB */)
{
    extern __shared__ __attribute__((aligned(16))) uint32_t smem[];
    constexpr int NSTEP = 4 * NCH;
    constexpr int NT = 64 * NWV, WPI = NT / 128, NIT = 8 * NCH / WPI;  // threads; plane words per row and pass; passes
    uint32_t *sA = smem;                                   // [NSTEP][64 lanes][4 dwords]
    float *s_sa = (float *)(smem + NSTEP * 256);           // [32] token scales
    float *s_sw = s_sa + 32;                               // [32 cbw] channel scales
    uint16_t *strips = (uint16_t *)(s_sw + 32 * cbw);      // [NWV wavefronts][FL_STRIP_HALFS]

    // the R workgroups of a strip sit 8 ids apart: same XCD, so the strip's second reader hits its L2
    const int nstrips = (g.M + 31) >> 5;
    const int id = blockIdx.x, kq = id >> 3;
    const int split = kq % R, strip_id = (kq / R) * 8 + (id & 7);
    if (strip_id >= nstrips) return;  // the grid is padded to rounds of 8 strips
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rw = g.rw;
    const int m0 = 32 * strip_id;
    const int cb0 = split * cbw;               // first channel block of this workgroup
    const int ncb = (g.N + 31) >> 5;           // channel blocks in all
    const int per_wave = cbw / NWV;            // channel blocks per wavefront, a multiple of FL_CB
    const int wcb0 = cb0 + wave * per_wave;    // first channel block of this wavefront

    // ---- requests, smallest first: scales, the strip's activations, the first group's weight bits
    const int quad = tid >> 2, j = tid & 3;
    const int row = quad & 31, m = m0 + row;
    const int mc = m < g.M ? m : 0;
    const bool have_sa = g.s_a.mode != 0 && g.s_a.ptr != nullptr;
    const uint16_t sa_bits = *(have_sa ? g.s_a.ptr + (g.s_a.mode == 1 ? 0 : mc) : A);
    const bool have_sw = g.s_w.mode != 0 && g.s_w.ptr != nullptr;
    constexpr int SW_PER = 2048 / NT;  // 2048 channel scales at most (cbw <= 64)
    uint16_t sw_bits[SW_PER];
#pragma unroll
    for (int i = 0; i < SW_PER; ++i) {
        const int n = 32 * cb0 + tid + NT * i;
        const bool want = tid + NT * i < 32 * cbw && n < g.N && have_sw;
        sw_bits[i] = *(want ? g.s_w.ptr + (g.s_w.mode == 1 ? 0 : n) : A);
    }
    uint4 x[NIT];
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int q = WPI * it + (quad >> 5), k0 = 32 * q + 8 * j;
        const bool inb = m < g.M && k0 < g.K;  // lanes outside re-read the first bytes and drop them
        x[it] = *(const uint4 *)(A + (inb ? (int64_t)m * lda + k0 : 0));
    }
    const int r32 = lane & 31, h = lane >> 5;
    uint4 wq[NCH][FL_CB];
    auto fetch_w = [&](int cb_first) {
#pragma unroll
        for (int c = 0; c < FL_CB; ++c) {
            int n = 32 * (cb_first + c) + r32;
            n = n < g.N ? n : g.N - 1;  // rows past the end are never stored
            const uint32_t *wrow = g.wsign + (int64_t)n * rw;
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch) {
                int kw = 8 * ch + 4 * h;
                kw = kw < rw ? kw : rw - 4;  // words past the end meet zero activations
                wq[ch][c] = *(const uint4 *)(wrow + kw);
            }
        }
    };
    fetch_w(wcb0);
    __builtin_amdgcn_sched_barrier(0);

    // ---- ternarise the strip into LDS
    const TernaryThr thr = ternary_thresholds(have_sa ? sa_bits : 0x3c00u, m < g.M);
    if ((quad >> 5) == 0 && j == 0) s_sa[row] = m < g.M ? (have_sa ? half_bits_to_float(sa_bits) : 1.0f) : 0.0f;
#pragma unroll
    for (int i = 0; i < SW_PER; ++i) {
        const int e = tid + NT * i, n = 32 * cb0 + e;
        if (e < 32 * cbw) s_sw[e] = n < g.N ? (have_sw ? half_bits_to_float(sw_bits[i]) : 1.0f) : 0.0f;
    }
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int q = WPI * it + (quad >> 5), k0 = 32 * q + 8 * j;
        uint4 v = x[it];
        if (!(m < g.M && k0 < g.K)) v = make_uint4(0, 0, 0, 0);
        const uint32_t D = fragment_dword(v, thr, j);
        const int jw = q & 7, step = 4 * (q >> 3) + (jw & 3), half = jw >> 2;
        sA[(step * 64 + half * 32 + row) * 4 + j] = D;
    }
    __syncthreads();

    // ---- products: no barrier from here on
    uint32_t m88 = 0x88888888u, c22 = 0x22222222u;
    asm volatile("" : "+s"(m88));
    asm volatile("" : "+v"(c22));
    uint16_t *strip = strips + wave * FL_STRIP_HALFS;
    const uint4 *sAl = (const uint4 *)sA + lane;
    for (int grp = 0; grp * FL_CB < per_wave; ++grp) {
        const int gcb = wcb0 + grp * FL_CB;
        if (gcb >= ncb) break;
        v16f acc[FL_CB][1];
#pragma unroll
        for (int c = 0; c < FL_CB; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[c][0][v] = 0.0f;
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch)
#pragma unroll
            for (int st = 0; st < 4; ++st) {
                const uint4 av = sAl[(4 * ch + st) * 64];
                v8i a;
                a[0] = (int)av.x; a[1] = (int)av.y; a[2] = (int)av.z; a[3] = (int)av.w;
                a[4] = a[5] = a[6] = a[7] = 0;
#pragma unroll
                for (int c = 0; c < FL_CB; ++c) {
                    const uint4 w4 = wq[ch][c];
                    const v8i b = widen_w(st == 0 ? w4.x : st == 1 ? w4.y : st == 2 ? w4.z : w4.w, m88, c22);
                    acc[c][0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b, a, acc[c][0], 4, 4, 0, 0, 0, 0);
                }
            }
        // the next group's bits are requested before this group's results are scaled and stored
        if ((grp + 1) * FL_CB < per_wave) fetch_w(gcb + FL_CB < ncb ? gcb + FL_CB : gcb);
        store_tile_fp16<1, FL_CB>(acc, g, s_sa, s_sw + 32 * (gcb - cb0), strip, m0, 32 * gcb, lane);
    }
}

// tuning settings: process-wide, read once per launch decision (relaxed atomics: any thread may set
// them while others launch; a launch sees either the old or the new value)
static std::atomic<int> g_linear_fused{1};  // 0: never; 1: where it pays; 2: wherever it can run; g_linear_fused_r > 0 forces the channel splits
static std::atomic<int> g_linear_fused_r{0};

}  // namespace


size_t gemm_fp4_frag_bytes(int M, int K)
{
    const int rw = 4 * ((K + 127) / 128);
    return (size_t)fp4_rb_pad(M) * fp4_s_pad(rw) * 1024;  // one KiB per (row block, k step)
}

// fp16 activations -> fragments (bwta_linear's first half on the FP4 path)
hipError_t launch_quantize_to_fp4(const void *A, int64_t lda, ScaleArg s_a, int M, int K, uint32_t *frag,
                                  hipStream_t st)
{
    const int rw = 4 * ((K + 127) / 128);
    const int rb_pad = fp4_rb_pad(M), s_pad = fp4_s_pad(rw);
    const int vec_ok = (((uintptr_t)A % 16) == 0 && (lda % 8) == 0 && (K % 8) == 0) ? 1 : 0;
    const int64_t units = (int64_t)s_pad * rb_pad;  // workgroups at one k step per thread
    if (units >= 4 * 2048)
        hipLaunchKernelGGL(k_quantize_to_fp4<4>, dim3((s_pad + 3) / 4, rb_pad), dim3(256), 0, st, (const uint16_t *)A, lda,
                           s_a, M, K, s_pad, frag, vec_ok);
    else if (units >= 2 * 2048)
        hipLaunchKernelGGL(k_quantize_to_fp4<2>, dim3((s_pad + 1) / 2, rb_pad), dim3(256), 0, st, (const uint16_t *)A, lda,
                           s_a, M, K, s_pad, frag, vec_ok);
    else
        hipLaunchKernelGGL(k_quantize_to_fp4<1>, dim3(s_pad, rb_pad), dim3(256), 0, st, (const uint16_t *)A, lda, s_a, M,
                           K, s_pad, frag, vec_ok);
    return hipGetLastError();
}

// One launch for the whole linear when K is short (see k_linear_fused).  The workgroups of a strip
// each ternarise it again and a weight operand feeds a single MFMA, so the kernel's cost grows
// faster with K than the two-kernel form's, while its fixed cost is 2 us lower.  Measured over
// M = 512 .. 16384, N = 768 .. 11008, K = 256 .. 1024 it is ahead everywhere for K <= 768 (by 5 to
// 40 %: 13.1 -> 10.4 us at 4096 x 3072 x 768, 17.8 -> 11.3 us at 16384 x 768 x 768) and for K = 1024
// up to N = 4096 and M = 8192; beyond, the two kernels win.
bool linear_fused_supported(const void *A, int64_t lda, const GemmArgs &g)
{
    const int mode = g_linear_fused.load(std::memory_order_relaxed);
    if (mode == 0) return false;
    const bool pays = g.K <= 768 || (g.N <= 4096 && g.M <= 8192);
    return (pays || mode == 2) && g.K <= 1024 && g.N >= 128 && g.out != nullptr &&
           g.acc == nullptr && ((uintptr_t)A % 16) == 0 && (lda % 8) == 0 && (g.K % 8) == 0;
}

hipError_t launch_linear_fused(const void *A, int64_t lda, const GemmArgs &g, hipStream_t st)
{
    const int nstrips = (g.M + 31) / 32, ncb = (g.N + 31) / 32;
    // Workgroups of 8 wavefronts (4 where a workgroup has fewer than 8 channel blocks) and as many
    // channel splits as make about 256 workgroups, i.e. two wavefronts per SIMD; at most 64 channel
    // blocks per workgroup.  Measured at M = 1024 .. 8192: against 4 wavefronts and twice the splits
    // the strip is ternarised half as often for the same number of wavefronts (10.3 against 11.7 us
    // at the benchmark's up layer, 16.3 against 20.3 us at M = 8192).  Groups of two channel blocks:
    // with several groups per wavefront the next group's weight bits arrive, and the other
    // wavefronts' MFMAs run, while a group is scaled and stored (groups of 4 were 1 us slower).
    int R = (256 + nstrips - 1) / nstrips;
    const int forced_r = g_linear_fused_r.load(std::memory_order_relaxed);
    if (forced_r > 0) R = forced_r;
    if (R > ncb) R = ncb;
    const int NWV = (ncb + R - 1) / R >= 8 ? 8 : 4;
    if (R < (ncb + 63) / 64) R = (ncb + 63) / 64;
    const int pw = ((ncb + R - 1) / R + NWV - 1) / NWV;  // channel blocks per wavefront
    const int CB = pw >= 2 ? 2 : 1;
    const int cbw = NWV * ((pw + CB - 1) / CB * CB);
    if (cbw > 64) return hipErrorInvalidValue;
    R = (ncb + cbw - 1) / cbw;
    const int nch = (g.rw + 7) / 8;
    const size_t smem = (size_t)nch * 4 * 1024 + (32 + 32 * cbw) * 4 + (size_t)NWV * FL_STRIP_HALFS * 2;
    const dim3 grid((unsigned)((nstrips + 7) / 8 * 8 * R)), block(64 * NWV);
#define BWTA_FL(N_, C_)                                                                                          \
    if (nch == N_ && CB == C_ && NWV == 4) {                                                                     \
        hipLaunchKernelGGL((k_linear_fused<N_, C_, 4>), grid, block, smem, st, (const uint16_t *)A, lda, g, R, cbw); \
        return hipGetLastError();                                                                                \
    }                                                                                                            \
    if (nch == N_ && CB == C_ && NWV == 8) {                                                                     \
        hipLaunchKernelGGL((k_linear_fused<N_, C_, 8>), grid, block, smem, st, (const uint16_t *)A, lda, g, R, cbw); \
        return hipGetLastError();                                                                                \
    }
    BWTA_FL(1, 1) BWTA_FL(1, 2) BWTA_FL(2, 1) BWTA_FL(2, 2) BWTA_FL(3, 1) BWTA_FL(3, 2) BWTA_FL(4, 1) BWTA_FL(4, 2)
#undef BWTA_FL
    return hipErrorInvalidValue;
}

void set_linear_fused(int mode, int r)
{
    g_linear_fused.store(mode, std::memory_order_relaxed);
    g_linear_fused_r.store(r, std::memory_order_relaxed);
}

// BWTA_Att with V^T prepared as fragments.  g: M = rows of V^T per batch entry (a multiple of 128),
// N = attention rows per entry, wsign = the boolean plane, s_a / s_w = the scales of V^T / of the
// attention operand, out = the context matrix [batch][N][ldo].
hipError_t launch_att_v_fp4(const GemmArgs &g, const uint32_t *frag, int batch, int64_t w_stride_words,
                            int64_t out_stride, float alpha, hipStream_t st)
{
    const int s_pad = fp4_s_pad(g.rw);
    const BatchArgs ba{(int64_t)(g.M / 32) * s_pad * 256, w_stride_words, out_stride, alpha, batch};
    return launch<2, 2, 2, 2, 2, false, 1, 8, 1>(g, frag, s_pad, st, batch, ba);
}

static std::atomic<int> g_fp4_tile{0};
void set_fp4_tile(int t) { g_fp4_tile.store(t, std::memory_order_relaxed); }

// frag_ready: the fragments were already produced by launch_quantize_to_fp4 (planes unused)
hipError_t launch_gemm_fp4(const GemmArgs &g, uint32_t *frag, bool frag_ready, hipStream_t st)
{
    const int rb_pad = fp4_rb_pad(g.M), s_pad = fp4_s_pad(g.rw);
    if (!frag_ready) {
        const int64_t wgs32 = (int64_t)((s_pad + 15) / 16) * rb_pad;  // workgroups at 32 words each
        if (wgs32 >= 1024)
            hipLaunchKernelGGL(k_planes_to_fp4<32>, dim3((s_pad + 15) / 16, rb_pad), dim3(256), 0, st, g.mask, g.sign, g.M,
                               g.K, g.rw, s_pad, frag);
        else if (2 * wgs32 >= 1024)
            hipLaunchKernelGGL(k_planes_to_fp4<16>, dim3((s_pad + 7) / 8, rb_pad), dim3(128), 0, st, g.mask, g.sign, g.M,
                               g.K, g.rw, s_pad, frag);
        else
            hipLaunchKernelGGL(k_planes_to_fp4<8>, dim3((s_pad + 3) / 4, rb_pad), dim3(64), 0, st, g.mask, g.sign, g.M,
                               g.K, g.rw, s_pad, frag);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    const int forced = g_fp4_tile.load(std::memory_order_relaxed);
    if ((forced == 223 || forced == 243 || forced == 323) && gemm_fp4_lds_supported(g))
        return launch_gemm_fp4_lds(g, frag, forced, st);
    // Large products: both operands through LDS by direct loads.  Measured against the register-fed
    // kernel below on ready fragments (us, M x N x K): 128 x 256 tiles of 8 wavefronts win once there are
    // about 160 of them and K is long enough to pay for filling the ring -- 2048 x 4096 x 4096 15.9 against
    // 18.2, 2048 x 11008 x 4096 40.4 against 48.7, 2048 x 4096 x 11008 37.4 against 43.3, 512 x 11008 x 4096
    // (172 tiles) 14.6 against 16.7, 8192 x 768 x 3072 (192) 12.1 against 13.8, 4096 x 4096 x 1024 12.6
    // against 14.8; with fewer, 128 x 128 tiles of 4 wavefronts win where they come to about one per compute
    // unit -- 1024 x 4096 x 4096 11.0 against 11.6, 512 x 8192 x 8192 17.7 against 19.0, 1024 x 4096 x 1024
    // 6.2 against 6.7 -- and lose below that (512 x 4096 x 4096: 10.6 against 8.8).
    if (forced == 0 && g.acc == nullptr && g.K >= 1024 && gemm_fp4_lds_supported(g)) {
        const int64_t tm = (g.M + 127) / 128;
        const int64_t tiles256 = tm * ((g.N + 255) / 256), tiles128 = tm * ((g.N + 127) / 128);
        if (tiles256 >= (g.K >= 2048 ? 160 : 224)) return launch_gemm_fp4_lds(g, frag, 243, st);
        if (tiles128 >= 224) return launch_gemm_fp4_lds(g, frag, 223, st);
    }
    if (g.acc) return launch<2, 2, 2, 2, 2, true>(g, frag, s_pad, st);  // int32 output: test / debug path
    switch (forced) {  // forced tile (tuning sweeps); 0 = heuristic below
    case 22: return launch<2, 2, 2, 2, 2, false>(g, frag, s_pad, st);
    case 23: return launch<2, 2, 2, 2, 3, false>(g, frag, s_pad, st);
    case 21: return launch<2, 1, 2, 2, 3, false>(g, frag, s_pad, st);
    case 12: return launch<1, 2, 2, 2, 3, false>(g, frag, s_pad, st);
    case 11: return launch<1, 1, 2, 2, 4, false>(g, frag, s_pad, st);
    case 13: return launch<1, 3, 4, 1, 2, false>(g, frag, s_pad, st);
    case 222: return launch<2, 2, 2, 2, 2, false, 2>(g, frag, s_pad, st);
    default: break;
    }
    // A few hundred tokens against a narrow matrix: 128 x 128 tiles would leave half the compute units
    // or more without a workgroup, 64 x 64 tiles quadruple the workgroups (measured at N = 4096,
    // 192-512 tokens: 7.5-9.4 us against 11.4-12.0 us at K = 4096, 15.8-19.7 against 24-25 at K = 11008).
    const int64_t tiles128 = (int64_t)((g.M + 127) / 128) * ((g.N + 127) / 128);
    if (tiles128 <= 128 && g.K >= 1024) return launch<1, 1, 2, 2, 4, false>(g, frag, s_pad, st);
    // Between 129 and 255 tiles of 128 x 128 some compute units get no workgroup at all.  If tiles of
    // 128 x 96 (four wavefronts of 32 x 96) number at most 256, every one of them still runs in the
    // first round and more compute units take part (measured at M = 4096, N = 768, K = 3072: 192 -> 256
    // workgroups, 9.7 -> 8.3 us).
    const int64_t tiles96 = (int64_t)((g.M + 127) / 128) * ((g.N + 95) / 96);
    if (tiles128 < 256 && tiles96 > tiles128 && tiles96 <= 256 && g.K >= 1024)
        return launch<1, 3, 4, 1, 2, false>(g, frag, s_pad, st);
    // measured: long K runs best with 2 wavefronts per SIMD (179 registers), short K with 3
    if (g.K >= 2048) return launch<2, 2, 2, 2, 2, false>(g, frag, s_pad, st);
    return launch<2, 2, 2, 2, 3, false>(g, frag, s_pad, st);
}

}  // namespace bwta
