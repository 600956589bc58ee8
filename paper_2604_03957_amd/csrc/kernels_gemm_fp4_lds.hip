// BWTA product on the FP4 matrix cores with BOTH operands staged through LDS by direct
// global->LDS loads (global_load_lds_dwordx4: 16 bytes per lane, no register in between).
//
// Why: with the activation fragments loaded straight into registers, each wavefront of a tile
// fetches its own copy of a fragment, and at 2 x 2 blocks of 32 x 32 per wavefront a compute unit
// running its matrix cores flat out would have to pull 64 bytes per clock through its vector memory
// path -- all of that path.  Here a fragment is fetched ONCE per workgroup into LDS and read from
// there by every wavefront that needs it (four of them on the widest tile), and the loads cost no
// VGPR, no LDS store instruction and (addresses being wave-uniform base + lane offset) no
// vector-ALU work.
//
// Layout and roles (Case 1 of the paper's arithmetic rules; operands exact in E2M1, sums exact in
// fp32, see kernels_gemm_fp4.hip):
//   * Workgroup tile (64 WAVES_M) tokens x (32 WN WAVES_N) channels; a wavefront owns 2 x WN blocks
//     of 32 x 32.
//   * K is walked in slabs of 256 (4 MFMA steps).  A slab of activations is 4 fragments of 1 KiB
//     per block of 32 tokens, already in operand order in memory, so one direct load per fragment
//     puts it into LDS exactly as a wavefront reads it back (16 bytes per lane, conflict-free).  A
//     slab of weights is 32 bytes per channel, 1 bit per weight; a direct load covers 32 channels
//     (lanes 0-31 fetch words 0..3 of their channel's 8, lanes 32-63 words 4..7), laid out so that
//     lane (r, h) of the MFMA finds the words of its four steps with two 8-byte reads.
//   * S stages of LDS form a ring; a slab is requested S - 1 iterations before it is used.  One
//     workgroup barrier per slab: before it every wavefront waits for ITS OWN requests of that slab
//     (s_waitcnt vmcnt(n): loads complete in order and every wavefront issues the same number per
//     slab, so n = the loads of the younger slabs still in flight); after it the slab is visible to
//     all, and the stage freed by the previous slab is requested again.  The last S - 1 slabs
//     request nothing (their n shrinks to 0).
//   * LDS reads are issued from inline assembly and waited for with explicit lgkmcnt counts: the
//     compiler cannot know which outstanding direct load an LDS read depends on and would otherwise
//     drain all of them (vmcnt(0)) in front of every read, serialising the ring.
//   * Epilogue as in the register-fed kernel (scale bits kept in two registers per thread through
//     the loop), with its LDS scratch in the S - 1 stages the last slab does not read: the scales
//     are parked there just before the last slab's barrier, the wavefronts' strips follow them, and
//     no wavefront waits for another between its last MFMA and its stores.
#include <type_traits>

#include "bwta_internal.h"
#include "bwta_fp4_tile.h"

namespace bwta {

namespace {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

constexpr int WM = 2;  // token blocks of 32 per wavefront

// f(integral_constant<T>), ..., f(integral_constant<N - 1>): a loop whose counter is a compile-time constant
template <int T, int N, class F>
__device__ __forceinline__ void static_for(const F &f)
{
    if constexpr (T < N) {
        f(std::integral_constant<int, T>{});
        static_for<T + 1, N>(f);
    }
}

template <int WN, int WAVES_M, int WAVES_N, int S>
struct LCfg {
    static constexpr int BM = 32 * WM * WAVES_M, BN = 32 * WN * WAVES_N;
    static constexpr int NW = WAVES_M * WAVES_N, THREADS = 64 * NW;
    static constexpr int AF = 4 * (BM / 32);             // activation fragments (1 KiB each) per slab
    static constexpr int WB = BN / 32;                   // blocks of 32 channels (1 KiB each) per slab
    static constexpr int A_BYTES = AF * 1024, STAGE_BYTES = (AF + WB) * 1024;  // a stage holds one slab
    static constexpr int A_ROUNDS = AF / NW, W_ROUNDS = WB / NW;  // direct loads per wavefront and slab
    static constexpr int LOADS = A_ROUNDS + W_ROUNDS;
    static constexpr int STRIP_HALFS = 32 * (32 * WN + 8);
    // epilogue scratch lives in the S - 1 stages the last slab does not use: scales and the first strips
    // in the first of them, the other strips in the following ones
    static constexpr int SCALE_BYTES = ((BN + BM) * 4 + 255) / 256 * 256;
    static constexpr int EPI_FIRST = (STAGE_BYTES - SCALE_BYTES) / (STRIP_HALFS * 2);
    static constexpr int EPI_PER_STAGE = STAGE_BYTES / (STRIP_HALFS * 2);
    static constexpr int SMEM_BYTES = S * STAGE_BYTES;
    static_assert(S >= 2 && EPI_FIRST + (S - 2) * EPI_PER_STAGE >= NW, "the free stages hold every wavefront's strip");
    static_assert(AF % NW == 0 && WB % NW == 0, "every wavefront issues the same loads per slab");
    static_assert(BN <= THREADS && BM <= THREADS, "one thread per scale");
    static_assert(SMEM_BYTES <= 160 * 1024, "LDS of one compute unit");
    static_assert(WN == 2 || WN == 4, "read schedules exist for 2 x 2 and 2 x 4 blocks per wavefront");
};

__device__ __forceinline__ void lds_direct_16(const void *src, uint32_t *lds_dst)
{
    __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1))) *)src,
                                     (void __attribute__((address_space(3))) *)lds_dst, 16, 0, 0);
}

// one MFMA step of a wavefront: WM token blocks x WN channel blocks
template <int WN>
__device__ __forceinline__ void mfma_step(v16f (&acc)[WN][WM], const u32x4 (&a)[WM], const uint32_t (&w)[WN], uint32_t m88,
                                          uint32_t c22)
{
    v8i vb[WN];
#pragma unroll
    for (int j = 0; j < WN; ++j) {
        vb[j] = widen_w(w[j], m88, c22);
    }
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            const v8i va = {(int)a[i].x, (int)a[i].y, (int)a[i].z, (int)a[i].w, 0, 0, 0, 0};
            acc[j][i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(vb[j], va, acc[j][i], 4, 4, 0, 0, 0, 0);
        }
}

#define BWTA_LDS_READ_A(dst, off) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(a_addr), "n"(off) : "memory")
#define BWTA_LDS_READ_W(dst, off) asm volatile("ds_read_b64 %0, %1 offset:%2" : "=v"(dst) : "v"(w_addr), "n"(off) : "memory")

// One slab (4 MFMA steps) of a wavefront: its LDS reads, in batches that the 4-bit counter can hold,
// each step waiting only for what it needs (LDS reads return in order), and its MFMAs.
// a_addr / w_addr: LDS byte addresses of this lane's first fragment / weight read in the stage.
template <int WN>
__device__ __forceinline__ void slab_compute(v16f (&acc)[WN][WM], uint32_t a_addr, uint32_t w_addr, uint32_t m88, uint32_t c22)
{
    u32x2 wlo[WN], whi[WN];
    if constexpr (WN == 4) {
        // 16 reads per slab (8 weight words, 8 fragments), one more than the counter holds: three batches
        u32x4 a0[2], a1[2], a2[2], a3[2];
        BWTA_LDS_READ_W(wlo[0], 0);
        BWTA_LDS_READ_W(wlo[1], 1024);
        BWTA_LDS_READ_W(wlo[2], 2048);
        BWTA_LDS_READ_W(wlo[3], 3072);
        BWTA_LDS_READ_A(a0[0], 0);
        BWTA_LDS_READ_A(a0[1], 4096);
        BWTA_LDS_READ_A(a1[0], 1024);
        BWTA_LDS_READ_A(a1[1], 5120);
        asm volatile("s_waitcnt lgkmcnt(2)"
                     : "+v"(wlo[0]), "+v"(wlo[1]), "+v"(wlo[2]), "+v"(wlo[3]), "+v"(a0[0]), "+v"(a0[1])::"memory");
        {
            const uint32_t w[4] = {wlo[0].x, wlo[1].x, wlo[2].x, wlo[3].x};
            mfma_step<4>(acc, a0, w, m88, c22);
        }
        __builtin_amdgcn_sched_barrier(0);
        BWTA_LDS_READ_W(whi[0], 512);
        BWTA_LDS_READ_W(whi[1], 1536);
        BWTA_LDS_READ_W(whi[2], 2560);
        BWTA_LDS_READ_W(whi[3], 3584);
        BWTA_LDS_READ_A(a2[0], 2048);
        BWTA_LDS_READ_A(a2[1], 6144);
        asm volatile("s_waitcnt lgkmcnt(6)" : "+v"(a1[0]), "+v"(a1[1])::"memory");
        {
            const uint32_t w[4] = {wlo[0].y, wlo[1].y, wlo[2].y, wlo[3].y};
            mfma_step<4>(acc, a1, w, m88, c22);
        }
        __builtin_amdgcn_sched_barrier(0);
        BWTA_LDS_READ_A(a3[0], 3072);
        BWTA_LDS_READ_A(a3[1], 7168);
        asm volatile("s_waitcnt lgkmcnt(2)"
                     : "+v"(whi[0]), "+v"(whi[1]), "+v"(whi[2]), "+v"(whi[3]), "+v"(a2[0]), "+v"(a2[1])::"memory");
        {
            const uint32_t w[4] = {whi[0].x, whi[1].x, whi[2].x, whi[3].x};
            mfma_step<4>(acc, a2, w, m88, c22);
        }
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a3[0]), "+v"(a3[1])::"memory");
        {
            const uint32_t w[4] = {whi[0].y, whi[1].y, whi[2].y, whi[3].y};
            mfma_step<4>(acc, a3, w, m88, c22);
        }
    } else {
        u32x4 a[4][2];
        // 12 reads in this order; each step waits until its own have returned (reads return in order)
        BWTA_LDS_READ_W(wlo[0], 0);
        BWTA_LDS_READ_W(wlo[1], 1024);
        BWTA_LDS_READ_A(a[0][0], 0);
        BWTA_LDS_READ_A(a[0][1], 4096);
        BWTA_LDS_READ_A(a[1][0], 1024);
        BWTA_LDS_READ_A(a[1][1], 5120);
        BWTA_LDS_READ_W(whi[0], 512);
        BWTA_LDS_READ_W(whi[1], 1536);
        BWTA_LDS_READ_A(a[2][0], 2048);
        BWTA_LDS_READ_A(a[2][1], 6144);
        BWTA_LDS_READ_A(a[3][0], 3072);
        BWTA_LDS_READ_A(a[3][1], 7168);
        // the values pass through the wait so that nothing that uses them can be scheduled above it
        asm volatile("s_waitcnt lgkmcnt(8)" : "+v"(wlo[0]), "+v"(wlo[1]), "+v"(a[0][0]), "+v"(a[0][1])::"memory");
        {
            const uint32_t w[2] = {wlo[0].x, wlo[1].x};
            mfma_step<2>(acc, a[0], w, m88, c22);
        }
        __builtin_amdgcn_sched_barrier(0);  // keep each step's MFMAs in front of the next wait
        asm volatile("s_waitcnt lgkmcnt(6)" : "+v"(a[1][0]), "+v"(a[1][1])::"memory");
        {
            const uint32_t w[2] = {wlo[0].y, wlo[1].y};
            mfma_step<2>(acc, a[1], w, m88, c22);
        }
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_waitcnt lgkmcnt(2)" : "+v"(whi[0]), "+v"(whi[1]), "+v"(a[2][0]), "+v"(a[2][1])::"memory");
        {
            const uint32_t w[2] = {whi[0].x, whi[1].x};
            mfma_step<2>(acc, a[2], w, m88, c22);
        }
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a[3][0]), "+v"(a[3][1])::"memory");
        {
            const uint32_t w[2] = {whi[0].y, whi[1].y};
            mfma_step<2>(acc, a[3], w, m88, c22);
        }
    }
}

// at least two wavefronts per SIMD whatever the workgroup size (two workgroups of four wavefronts
// share a compute unit): the register budget is 256, not 512
template <int WN, int WAVES_M, int WAVES_N, int S, bool WITH_ACC>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) __attribute__((amdgpu_waves_per_eu(2)))
void k_gemm_fp4_lds(GemmArgs g, const uint32_t *__restrict__ frag, int s_pad, int tiles_n, int tiles_total)
{
    using C = LCfg<WN, WAVES_M, WAVES_N, S>;
    extern __shared__ __attribute__((aligned(1024))) uint32_t smem[];
    int tm, tn;
    tile_of_workgroup(tiles_n, tiles_total, tm, tn);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform by construction: keeps addressing scalar
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int r32 = lane & 31, h = lane >> 5;
    const int m0 = tm * C::BM, n0 = tn * C::BN;
    const int rw = g.rw;
    const int nslab = s_pad >> 2;  // slabs of 4 steps; the fragment buffer is padded to 8 steps

    // ---- scale bits: requested first, kept in registers through the loop
    const bool want_sw = tid < C::BN && n0 + tid < g.N, want_sa = tid < C::BM && m0 + tid < g.M;
    const bool have_sw = want_sw && g.s_w.mode != 0 && g.s_w.ptr != nullptr;
    const bool have_sa = want_sa && g.s_a.mode != 0 && g.s_a.ptr != nullptr;
    const uint16_t *scale_safe = (const uint16_t *)g.wsign;
    const uint16_t sw_bits = *(have_sw ? g.s_w.ptr + (g.s_w.mode == 1 ? 0 : n0 + tid) : scale_safe);
    const uint16_t sa_bits = *(have_sa ? g.s_a.ptr + (g.s_a.mode == 1 ? 0 : m0 + tid) : scale_safe);

    // ---- what this wavefront requests per slab.  Round q of the activation part: fragment f = q NW +
    // wave (token block f / 4, step f % 4).  Round q of the weight part: channel block q NW + wave; lane
    // (r, p) fetches words 4 p .. 4 p + 3 of its channel's 8.  Sources are a wave-uniform base plus a
    // 32-bit lane offset.
    const char *a_tile = (const char *)frag + (int64_t)tm * (C::BM / 32) * s_pad * 1024;
    const uint32_t a_lane = (uint32_t)lane * 16u;
    uint32_t w_lane[C::W_ROUNDS];  // byte offset of this lane's channel row from the weights' base, plus its half
#pragma unroll
    for (int q = 0; q < C::W_ROUNDS; ++q) {
        int row = n0 + 32 * (q * C::NW + wave) + r32;
        row = row < g.N ? row : g.N - 1;  // channels past the end are never stored
        w_lane[q] = (uint32_t)row * (uint32_t)rw * 4u + 16u * (uint32_t)h;
    }
    const uint32_t w_last = (uint32_t)(rw - 4) * 4u - 16u * (uint32_t)h;  // added to a row's offset: its last four words
    auto request = [&](int slab, int stage) {
        uint32_t *st = smem + stage * (C::STAGE_BYTES / 4);
#pragma unroll
        for (int q = 0; q < C::A_ROUNDS; ++q) {
            const int f = q * C::NW + wave;
            const char *src = a_tile + ((int64_t)(f >> 2) * s_pad + 4 * slab + (f & 3)) * 1024;
            lds_direct_16(src + a_lane, st + f * 256);
        }
#pragma unroll
        for (int q = 0; q < C::W_ROUNDS; ++q) {
            // words 8 slab + 4 p .. + 3; past the row's end (K tail) the last four instead: if the slab's
            // first half still exists those ARE its words, and whatever lies beyond meets zero activations
            const bool inside = 8 * slab + 8 <= rw;
            const uint32_t off = inside ? w_lane[q] + 32u * (uint32_t)slab : w_lane[q] + w_last;
            lds_direct_16((const char *)g.wsign + off, st + C::A_BYTES / 4 + (q * C::NW + wave) * 256);
        }
    };

    v16f acc[WN][WM];  // [channel block][token block]
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
        for (int i = 0; i < WM; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][i][v] = 0.0f;

    uint32_t m88 = 0x88888888u, c22 = 0x22222222u;
    asm volatile("" : "+s"(m88));
    asm volatile("" : "+v"(c22));

#pragma unroll
    for (int s = 0; s < S - 1; ++s) request(s < nslab ? s : nslab - 1, s);

    // LDS byte addresses of this lane's reads inside a stage
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint32_t *)smem;
    const uint32_t a_rd = lds0 + (uint32_t)((wm * WM) * 4096 + lane * 16);                          // + i 4096 + step 1024
    const uint32_t w_rd = lds0 + (uint32_t)(C::A_BYTES + (wn * WN) * 1024 + r32 * 16 + h * 8);      // + j 1024 (+ 512: steps 2, 3)

    // Inside the slab loop a wavefront issues ahead of the wavefronts of the other workgroup on this
    // compute unit that are still setting up or already in their epilogue (scalar address arithmetic,
    // conversions, LDS strips): those fill the gaps.  Measured on the shape that runs several rounds of
    // workgroups per compute unit (2048 x 11008 x 4096): 45.0 -> 43.1 us on the same box; no change on
    // the single-round shapes.
    __builtin_amdgcn_s_setprio(3);
    int stage = 0;
    // One slab: wait for the own requests of it (YOUNGER slabs of this wavefront may stay in flight: loads
    // complete in order and every wavefront issues LOADS per slab), then the barrier after which everyone's
    // have landed and everyone is done reading the previous slab.
    auto slab = [&](auto younger, auto before_barrier, auto after_barrier) {
        __builtin_amdgcn_sched_barrier(0);  // the previous slab's MFMAs stay in front of the wait
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(decltype(younger)::value * C::LOADS) : "memory");
        before_barrier();
        __builtin_amdgcn_s_barrier();
        after_barrier();
        const uint32_t a_addr = a_rd + (uint32_t)(stage * C::STAGE_BYTES), w_addr = w_rd + (uint32_t)(stage * C::STAGE_BYTES);
        stage = stage + 1 == S ? 0 : stage + 1;
        slab_compute<WN>(acc, a_addr, w_addr, m88, c22);
    };
    auto nothing = [] {};
    // slabs that still have a successor S - 1 ahead: request it into the stage the previous slab was read from
    for (int it = 0; it + S - 1 < nslab; ++it)
        slab(std::integral_constant<int, S - 2>{}, nothing, [&] {
            int st_n = stage + S - 1;
            st_n = st_n >= S ? st_n - S : st_n;
            request(it + S - 1, st_n);
        });
    // The last S - 1 slabs request nothing: ever fewer loads stay in flight, and the stages they would
    // have filled are free.  The stage behind the last slab's takes the scales (written before the last
    // barrier, which publishes them); it and the one after it take the wavefronts' epilogue strips.  So a
    // wavefront goes from its last MFMA into its epilogue without waiting for anyone.
    float *sc_lds = nullptr;  // [BN] channel scales, then [BM] token scales
    static_for<0, S - 1>([&](auto t) {
        constexpr int T = decltype(t)::value;  // the slab nslab - (S - 1) + T; S - 2 - T younger ones in flight
        if constexpr (T < S - 2)
            slab(std::integral_constant<int, S - 2 - T>{}, nothing, nothing);
        else
            slab(std::integral_constant<int, 0>{},
                 [&] {
                     const int st_f = stage + 1 == S ? 0 : stage + 1;
                     sc_lds = (float *)(smem + st_f * (C::STAGE_BYTES / 4));
                     if (tid < C::BN) sc_lds[tid] = have_sw ? half_bits_to_float(sw_bits) : (want_sw ? 1.0f : 0.0f);
                     if (tid < C::BM) sc_lds[C::BN + tid] = have_sa ? half_bits_to_float(sa_bits) : (want_sa ? 1.0f : 0.0f);
                 },
                 nothing);
    });
    __builtin_amdgcn_s_setprio(0);
    // `stage` now names the stage behind the last slab's; wavefronts 0 .. EPI_FIRST - 1 put their strips
    // behind the scales, the others into the stages that follow
    int st_e = stage;
    int slot = wave;
    uint32_t strip_off = C::SCALE_BYTES;
    if (wave >= C::EPI_FIRST) {
        slot = wave - C::EPI_FIRST;
        st_e = stage + 1 + slot / C::EPI_PER_STAGE;
        st_e = st_e >= S ? st_e - S : st_e;
        slot = slot % C::EPI_PER_STAGE;
        strip_off = 0;
    }

    const int m_wave = m0 + wm * WM * 32, n_wave = n0 + wn * WN * 32;
    if (WITH_ACC && g.acc) {
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
    uint16_t *strip = (uint16_t *)((char *)smem + st_e * C::STAGE_BYTES + strip_off) + slot * C::STRIP_HALFS;
    store_tile_fp16<WM, WN>(acc, g, sc_lds + C::BN + wm * WM * 32, sc_lds + wn * WN * 32, strip, m_wave, n_wave, lane);
}

#undef BWTA_LDS_READ_A
#undef BWTA_LDS_READ_W

template <int WN, int WAVES_M, int WAVES_N, int S, bool WITH_ACC>
hipError_t launch_lds(const GemmArgs &g, const uint32_t *frag, int s_pad, hipStream_t st)
{
    using C = LCfg<WN, WAVES_M, WAVES_N, S>;
    static bool configured = false;  // benign race: setting the attribute twice is harmless
    if (!configured) {
        hipError_t e = hipFuncSetAttribute((const void *)k_gemm_fp4_lds<WN, WAVES_M, WAVES_N, S, WITH_ACC>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, C::SMEM_BYTES);
        if (e != hipSuccess) return e;
        configured = true;
    }
    if ((s_pad >> 2) < S - 1) return hipErrorInvalidValue;  // the kernel's tail runs S - 1 slabs (the padding gives 2)
    const int tiles_n = (g.N + C::BN - 1) / C::BN, tiles_m = (g.M + C::BM - 1) / C::BM;
    const int64_t total = (int64_t)tiles_n * tiles_m;
    if (total > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL((k_gemm_fp4_lds<WN, WAVES_M, WAVES_N, S, WITH_ACC>), dim3((unsigned)total), dim3(C::THREADS),
                       C::SMEM_BYTES, st, g, frag, s_pad, tiles_n, (int)total);
    return hipGetLastError();
}

}  // namespace

// byte offsets into the packed weights are 32 bits in this kernel
bool gemm_fp4_lds_supported(const GemmArgs &g) { return (int64_t)g.N * g.rw * 4 <= 0xffffffffll && g.rw >= 4; }

// The LDS-staged tiled kernel on ready fragments.  variant: 243 = 128 x 256 tiles, 8 wavefronts of
// 64 x 64 (the dispatcher's choice); 223 = 128 x 128 tiles, 4 wavefronts of 64 x 64; 323 = 128 x 256
// tiles, 4 wavefronts of 64 tokens x 128 channels; all with a ring of three slabs.
hipError_t launch_gemm_fp4_lds(const GemmArgs &g, const uint32_t *frag, int variant, hipStream_t st)
{
    const int s_pad = fp4_s_pad(g.rw);
    if (!gemm_fp4_lds_supported(g)) return hipErrorInvalidValue;
#define BWTA_LDS_CASE(ID, WN, WVM, WVN, S)                                       \
    case ID:                                                                     \
        return g.acc ? launch_lds<WN, WVM, WVN, S, true>(g, frag, s_pad, st)     \
                     : launch_lds<WN, WVM, WVN, S, false>(g, frag, s_pad, st);
    switch (variant) {
        BWTA_LDS_CASE(223, 2, 2, 2, 3)
        BWTA_LDS_CASE(243, 2, 2, 4, 3)
        BWTA_LDS_CASE(323, 4, 2, 2, 3)
    default: return hipErrorInvalidValue;
    }
#undef BWTA_LDS_CASE
}

}  // namespace bwta
