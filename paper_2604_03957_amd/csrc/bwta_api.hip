// C ABI of libbwta.so: host-side argument validation and dispatch.  Every check happens before
// anything is enqueued, so a bad call never touches the device.
#include "../../include/bwta.h"
#include "../../include/bwta_tuning.h"

#include <atomic>
#include <mutex>

#include "bwta_internal.h"

// Scratch of the entry point that allocates nothing (bwta_linear_static): part of the library's
// image on every GPU it runs on, until the process ends.  In host code this name is only a handle
// for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[BWTA_STATIC_SCRATCH_BYTES];

namespace {

// the array's address on each device, looked up once per device with that device current
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

int static_scratch_ptr(void **out, hipError_t *err)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess && (dev < 0 || dev >= kMaxDevices)) e = hipErrorInvalidDevice;
    if (e == hipSuccess) {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[dev]) {
            void *p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e == hipSuccess && !p) e = hipErrorInvalidSymbol;
            if (e == hipSuccess) g_scratch_ptr[dev] = p;
        }
        if (e == hipSuccess) *out = g_scratch_ptr[dev];
    }
    *err = e;
    return e == hipSuccess ? BWTA_OK : BWTA_ERR_HIP;
}

std::atomic<int> g_path{BWTA_PATH_AUTO};
thread_local int t_last_hip_error = 0;

inline bool aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int hip_result(hipError_t e)
{
    if (e == hipSuccess) return BWTA_OK;
    t_last_hip_error = (int)e;
    return BWTA_ERR_HIP;
}

bool scale_mode_ok(int mode) { return mode >= BWTA_SCALE_NONE && mode <= BWTA_SCALE_VECTOR; }

size_t plane_bytes(int M, int K) { return round_up((size_t)M * (size_t)bwta_plane_row_words(K) * 4u, 256); }

int resolve_path(int M, int N, int K)
{
    int p = g_path.load(std::memory_order_relaxed);
    return p == BWTA_PATH_AUTO ? bwta_auto_path(M, N, K) : p;  // AUTO depends on M only
}

// the FP4 path consumes activation fragments (prefill kernel) unless the shape is decode-sized, in
// which case the matrix-core decode kernel reads the canonical planes directly
bool fp4_uses_fragments(int M, int K)
{
    bwta::GemmArgs g{};
    g.M = M;
    g.N = 1;
    g.K = K;
    g.rw = (int)(4 * (((int64_t)K + 127) / 128));
    return resolve_path(M, 1, K) == BWTA_PATH_FP4 && !bwta::gemv_fp4_supported(g);
}

// Which kernel computes a product from canonical planes.  The tiled FP4 kernel is the only one that
// needs scratch (it converts the planes into fragments first); when no scratch comes with the call
// (have_scratch false: the operand was prepared as planes by an earlier call) a shape that would
// take it runs on the int8 matrix-core kernel or the popcount kernels instead, which read planes
// directly and give the same bits.
int plan_from_planes(const bwta::GemmArgs &g, bool have_scratch)
{
    const int path = resolve_path(g.M, g.N, g.K);
    if (path == BWTA_PATH_FP4 && bwta::gemv_fp4_supported(g)) return BWTA_KERNEL_GEMV_FP4;
    if (path == BWTA_PATH_FP4 && have_scratch) return BWTA_KERNEL_GEMM_FP4;
    if ((path == BWTA_PATH_MFMA || path == BWTA_PATH_FP4) && bwta::gemm_mfma_supported(g)) return BWTA_KERNEL_GEMM_MFMA_I8;
    if (bwta::gemv_popc_supported(g)) return BWTA_KERNEL_GEMV_POPC;
    return BWTA_KERNEL_GEMM_POPC;
}

// workspace layout: [mask planes | sign planes | FP4 activation fragments]
int run_gemm(const bwta::GemmArgs &g, void *workspace, hipStream_t st)
{
    switch (plan_from_planes(g, workspace != nullptr)) {
    case BWTA_KERNEL_GEMV_FP4: return hip_result(bwta::launch_gemv_fp4(g, st));
    case BWTA_KERNEL_GEMM_FP4: {
        uint32_t *frag = (uint32_t *)((char *)workspace + 2 * plane_bytes(g.M, g.K));
        return hip_result(bwta::launch_gemm_fp4(g, frag, false, st));
    }
    case BWTA_KERNEL_GEMM_MFMA_I8: return hip_result(bwta::launch_gemm_mfma(g, st));
    case BWTA_KERNEL_GEMV_POPC: return hip_result(bwta::launch_gemv_popc(g, st));
    default: return hip_result(bwta::launch_gemm_popc(g, st));
    }
}

}  // namespace

extern "C" {

int64_t bwta_plane_row_words(int K) { return K <= 0 ? 0 : 4 * (((int64_t)K + 127) / 128); }

size_t bwta_workspace_bytes(int M, int N, int K)
{
    if (M <= 0 || N <= 0 || K <= 0) return 0;
    // mask + sign planes of bwta_linear, then the FP4 activation fragments of the FP4 kernel
    return 2 * plane_bytes(M, K) + round_up(bwta::gemm_fp4_frag_bytes(M, K), 256);
}

int bwta_quantize_pack_act(const void *A, int a_dtype, int64_t lda, const void *s_a, int scale_mode,
                           int M, int K, uint32_t *mask, uint32_t *sign, int32_t *nnz,
                           bwta_stream_t stream)
{
    if (a_dtype != BWTA_DTYPE_FP16 && a_dtype != BWTA_DTYPE_INT8) return BWTA_ERR_UNSUPPORTED;
    if (!scale_mode_ok(scale_mode)) return BWTA_ERR_UNSUPPORTED;
    if (M < 0 || K < 0 || (M > 0 && K == 0)) return BWTA_ERR_SHAPE;
    if (M == 0) return BWTA_OK;
    if (lda < K) return BWTA_ERR_SHAPE;
    if (!A || !mask || !sign) return BWTA_ERR_NULL;
    if (scale_mode != BWTA_SCALE_NONE && a_dtype == BWTA_DTYPE_FP16 && !s_a) return BWTA_ERR_NULL;
    if (!aligned(mask, 16) || !aligned(sign, 16)) return BWTA_ERR_ALIGN;
    if (a_dtype == BWTA_DTYPE_FP16 && !aligned(A, 2)) return BWTA_ERR_ALIGN;
    if (s_a && !aligned(s_a, 2)) return BWTA_ERR_ALIGN;
    if (nnz && !aligned(nnz, 4)) return BWTA_ERR_ALIGN;
    bwta::ScaleArg sa{(const uint16_t *)s_a, s_a ? scale_mode : BWTA_SCALE_NONE};
    return hip_result(bwta::launch_quantize_pack(A, a_dtype, lda, sa, M, K, mask, sign, nnz, (hipStream_t)stream));
}

int bwta_pack_weights(const void *W, int w_dtype, int64_t ldw, int N, int K, uint32_t *wsign,
                      bwta_stream_t stream)
{
    if (w_dtype != BWTA_DTYPE_FP16 && w_dtype != BWTA_DTYPE_INT8) return BWTA_ERR_UNSUPPORTED;
    if (N < 0 || K < 0 || (N > 0 && K == 0)) return BWTA_ERR_SHAPE;
    if (N == 0) return BWTA_OK;
    if (ldw < K) return BWTA_ERR_SHAPE;
    if (!W || !wsign) return BWTA_ERR_NULL;
    if (!aligned(wsign, 16)) return BWTA_ERR_ALIGN;
    if (w_dtype == BWTA_DTYPE_FP16 && !aligned(W, 2)) return BWTA_ERR_ALIGN;
    return hip_result(bwta::launch_pack_weights(W, w_dtype, ldw, N, K, wsign, (hipStream_t)stream));
}

static int check_gemm_common(int M, int N, int K, const void *s_a, int a_mode, const void *s_w, int w_mode,
                             const void *out, int64_t ldo)
{
    if (!scale_mode_ok(a_mode) || !scale_mode_ok(w_mode)) return BWTA_ERR_UNSUPPORTED;
    if (M < 0 || N < 0 || K < 0 || (M > 0 && N > 0 && K == 0)) return BWTA_ERR_SHAPE;
    if (out && ldo < N) return BWTA_ERR_SHAPE;
    if (a_mode != BWTA_SCALE_NONE && !s_a) return BWTA_ERR_NULL;
    if (w_mode != BWTA_SCALE_NONE && !s_w) return BWTA_ERR_NULL;
    if ((s_a && !aligned(s_a, 2)) || (s_w && !aligned(s_w, 2))) return BWTA_ERR_ALIGN;
    if (out && !aligned(out, 2)) return BWTA_ERR_ALIGN;
    return BWTA_OK;
}

int bwta_gemm(const uint32_t *mask, const uint32_t *sign, const uint32_t *wsign, int M, int N, int K,
              const void *s_a, int a_scale_mode, const void *s_w, int w_scale_mode, int32_t *acc,
              void *out, int64_t ldo, void *workspace, size_t workspace_bytes, bwta_stream_t stream)
{
    int rc = check_gemm_common(M, N, K, s_a, a_scale_mode, s_w, w_scale_mode, out, ldo);
    if (rc != BWTA_OK) return rc;
    if (M == 0 || N == 0) return BWTA_OK;
    if (!sign || !wsign) return BWTA_ERR_NULL;
    if (!acc && !out) return BWTA_ERR_NULL;
    if ((mask && !aligned(mask, 16)) || !aligned(sign, 16) || !aligned(wsign, 16)) return BWTA_ERR_ALIGN;
    if (acc && !aligned(acc, 4)) return BWTA_ERR_ALIGN;
    if (!workspace || workspace_bytes < bwta_workspace_bytes(M, N, K)) return BWTA_ERR_WORKSPACE;
    if (!aligned(workspace, 256)) return BWTA_ERR_ALIGN;
    // binary (+-1) activations: the W1A1 layer.  Every element is non-zero.  The tiled matrix-core
    // path synthesises the mask while it converts the sign plane (no mask plane is written or read);
    // the other kernels get a full mask built in the workspace, whose mask area is otherwise unused here.
    if (!mask && !fp4_uses_fragments(M, K)) {
        int rcm = hip_result(bwta::launch_full_mask((uint32_t *)workspace, M, K, (hipStream_t)stream));
        if (rcm != BWTA_OK) return rcm;
        mask = (const uint32_t *)workspace;
    }
    bwta::GemmArgs g{mask, sign, wsign, M, N, K, (int)bwta_plane_row_words(K),
                     {(const uint16_t *)s_a, s_a ? a_scale_mode : BWTA_SCALE_NONE},
                     {(const uint16_t *)s_w, s_w ? w_scale_mode : BWTA_SCALE_NONE},
                     acc, (uint16_t *)out, ldo};
    return run_gemm(g, workspace, (hipStream_t)stream);
}

int bwta_linear(const void *A, int64_t lda, const void *s_a, int a_scale_mode, const uint32_t *wsign,
                const void *s_w, int w_scale_mode, int M, int N, int K, void *out, int64_t ldo,
                void *workspace, size_t workspace_bytes, bwta_stream_t stream)
{
    int rc = check_gemm_common(M, N, K, s_a, a_scale_mode, s_w, w_scale_mode, out, ldo);
    if (rc != BWTA_OK) return rc;
    if (M == 0 || N == 0) return BWTA_OK;
    if (lda < K) return BWTA_ERR_SHAPE;
    if (!A || !wsign || !out) return BWTA_ERR_NULL;
    if (!aligned(A, 2) || !aligned(wsign, 16)) return BWTA_ERR_ALIGN;
    if (!workspace || workspace_bytes < bwta_workspace_bytes(M, N, K)) return BWTA_ERR_WORKSPACE;
    if (!aligned(workspace, 256)) return BWTA_ERR_ALIGN;
    if (resolve_path(M, N, K) == BWTA_PATH_FP4) {
        bwta::GemmArgs g{nullptr, nullptr, wsign, M, N, K, (int)bwta_plane_row_words(K),
                         {(const uint16_t *)s_a, s_a ? a_scale_mode : BWTA_SCALE_NONE},
                         {(const uint16_t *)s_w, s_w ? w_scale_mode : BWTA_SCALE_NONE},
                         nullptr, (uint16_t *)out, ldo};
        if (bwta::linear_fused_supported(A, lda, g))
            return hip_result(bwta::launch_linear_fused(A, lda, g, (hipStream_t)stream));
    }
    int format = 0;
    rc = bwta_prepare_act(A, lda, s_a, a_scale_mode, M, K, workspace, workspace_bytes, &format, stream);
    if (rc != BWTA_OK) return rc;
    return bwta_gemm_prepared(workspace, workspace_bytes, format, wsign, M, N, K, s_a, a_scale_mode, s_w,
                              w_scale_mode, nullptr, out, ldo, stream);
}

int bwta_prepared_format(int M, int K)
{
    if (M <= 0 || K <= 0) return BWTA_PREPARED_PLANES;
    return fp4_uses_fragments(M, K) ? BWTA_PREPARED_FP4 : BWTA_PREPARED_PLANES;
}

size_t bwta_static_scratch_bytes(void) { return BWTA_STATIC_SCRATCH_BYTES; }

int bwta_static_scratch_init(void)
{
    void *p = nullptr;
    hipError_t e;
    int rc = static_scratch_ptr(&p, &e);
    if (rc != BWTA_OK) t_last_hip_error = (int)e;
    return rc;
}

int bwta_linear_static(const void *A, int64_t lda, const void *s_a, int a_scale_mode, const uint32_t *wsign,
                       const void *s_w, int w_scale_mode, int M, int N, int K, void *out, int64_t ldo,
                       bwta_stream_t stream)
{
    // the shape must fit before anything else is looked at: a caller sizing its batches to the limit
    // gets this answer whatever else is wrong with the call
    if (M > 0 && N > 0 && K > 0 && bwta_workspace_bytes(M, N, K) > BWTA_STATIC_SCRATCH_BYTES) return BWTA_ERR_TOO_LARGE;
    void *ws = nullptr;
    if (M > 0 && N > 0 && K > 0) {
        hipError_t e;
        int rc = static_scratch_ptr(&ws, &e);
        if (rc != BWTA_OK) {
            t_last_hip_error = (int)e;
            return rc;
        }
    }
    // Nothing in the scratch has to start from zero: the ternarisation kernels write every word the
    // product kernels read (padding rows and k steps included), so the previous call's contents are
    // simply overwritten.
    return bwta_linear(A, lda, s_a, a_scale_mode, wsign, s_w, w_scale_mode, M, N, K, out, ldo, ws,
                       ws ? (size_t)BWTA_STATIC_SCRATCH_BYTES : 0, stream);
}

size_t bwta_prepared_bytes(int M, int K)
{
    if (M <= 0 || K <= 0) return 0;
    return 2 * plane_bytes(M, K) + round_up(bwta::gemm_fp4_frag_bytes(M, K), 256);
}

int bwta_prepare_act(const void *A, int64_t lda, const void *s_a, int a_scale_mode, int M, int K,
                     void *prepared, size_t prepared_bytes, int *prepared_format, bwta_stream_t stream)
{
    if (!scale_mode_ok(a_scale_mode)) return BWTA_ERR_UNSUPPORTED;
    if (M < 0 || K < 0 || (M > 0 && K == 0)) return BWTA_ERR_SHAPE;
    if (!prepared_format) return BWTA_ERR_NULL;
    *prepared_format = bwta_prepared_format(M, K);  // decided once, here; the consumer is told, it does not re-derive it
    if (M == 0) return BWTA_OK;
    if (lda < K) return BWTA_ERR_SHAPE;
    if (!A) return BWTA_ERR_NULL;
    if (a_scale_mode != BWTA_SCALE_NONE && !s_a) return BWTA_ERR_NULL;
    if (!aligned(A, 2) || (s_a && !aligned(s_a, 2))) return BWTA_ERR_ALIGN;
    if (!prepared || prepared_bytes < bwta_prepared_bytes(M, K)) return BWTA_ERR_WORKSPACE;
    if (!aligned(prepared, 256)) return BWTA_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    bwta::ScaleArg sa{(const uint16_t *)s_a, s_a ? a_scale_mode : BWTA_SCALE_NONE};
    if (*prepared_format == BWTA_PREPARED_FP4) {
        uint32_t *frag = (uint32_t *)((char *)prepared + 2 * plane_bytes(M, K));
        return hip_result(bwta::launch_quantize_to_fp4(A, lda, sa, M, K, frag, st));
    }
    uint32_t *mask = (uint32_t *)prepared;
    uint32_t *sign = (uint32_t *)((char *)prepared + plane_bytes(M, K));
    return hip_result(bwta::launch_quantize_pack(A, BWTA_DTYPE_FP16, lda, sa, M, K, mask, sign, nullptr, st));
}

int bwta_prepare_act_autoscale(const void *A, int64_t lda, int M, int K, void *s_a, void *prepared,
                               size_t prepared_bytes, int *prepared_format, bwta_stream_t stream)
{
    if (M < 0 || K < 0 || (M > 0 && K == 0)) return BWTA_ERR_SHAPE;
    if (!prepared_format) return BWTA_ERR_NULL;
    *prepared_format = bwta_prepared_format(M, K);
    if (M == 0) return BWTA_OK;
    if (lda < K) return BWTA_ERR_SHAPE;
    if (K > 32768) return BWTA_ERR_UNSUPPORTED;  // a token row is held in one workgroup's registers
    if (!A || !s_a) return BWTA_ERR_NULL;
    if (!aligned(A, 2) || !aligned(s_a, 2)) return BWTA_ERR_ALIGN;
    if (!prepared || prepared_bytes < bwta_prepared_bytes(M, K)) return BWTA_ERR_WORKSPACE;
    if (!aligned(prepared, 256)) return BWTA_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    uint32_t *mask = (uint32_t *)prepared;
    uint32_t *sign = (uint32_t *)((char *)prepared + plane_bytes(M, K));
    uint32_t *frag =
        *prepared_format == BWTA_PREPARED_FP4 ? (uint32_t *)((char *)prepared + 2 * plane_bytes(M, K)) : nullptr;
    return hip_result(bwta::launch_act_scale_quantize(A, lda, M, K, (uint16_t *)s_a, frag, mask, sign, st));
}

int bwta_gemm_prepared(const void *prepared, size_t prepared_bytes, int prepared_format, const uint32_t *wsign,
                       int M, int N, int K, const void *s_a, int a_scale_mode, const void *s_w, int w_scale_mode,
                       int32_t *acc, void *out, int64_t ldo, bwta_stream_t stream)
{
    int rc = check_gemm_common(M, N, K, s_a, a_scale_mode, s_w, w_scale_mode, out, ldo);
    if (rc != BWTA_OK) return rc;
    if (prepared_format != BWTA_PREPARED_PLANES && prepared_format != BWTA_PREPARED_FP4) return BWTA_ERR_UNSUPPORTED;
    if (M == 0 || N == 0) return BWTA_OK;
    if (!wsign) return BWTA_ERR_NULL;
    if (!acc && !out) return BWTA_ERR_NULL;
    if (!aligned(wsign, 16) || (acc && !aligned(acc, 4))) return BWTA_ERR_ALIGN;
    if (!prepared || prepared_bytes < bwta_prepared_bytes(M, K)) return BWTA_ERR_WORKSPACE;
    if (!aligned(prepared, 256)) return BWTA_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    const uint32_t *mask = (const uint32_t *)prepared;
    const uint32_t *sign = (const uint32_t *)((const char *)prepared + plane_bytes(M, K));
    bwta::GemmArgs g{mask, sign, wsign, M, N, K, (int)bwta_plane_row_words(K),
                     {(const uint16_t *)s_a, s_a ? a_scale_mode : BWTA_SCALE_NONE},
                     {(const uint16_t *)s_w, s_w ? w_scale_mode : BWTA_SCALE_NONE},
                     acc, (uint16_t *)out, ldo};
    // The operand's format, not the current path setting, says which kernels can read it: fragments go
    // to the tiled FP4 kernel; planes go to a kernel that reads planes and needs no scratch.
    if (prepared_format == BWTA_PREPARED_FP4) {
        uint32_t *frag = (uint32_t *)((char *)prepared + 2 * plane_bytes(M, K));
        return hip_result(bwta::launch_gemm_fp4(g, frag, true, st));
    }
    return run_gemm(g, nullptr, st);
}

int bwta_gemm_grouped(const bwta_gemm_problem *problems, int count, int M, int N, int K, int a_scale_mode,
                      int w_scale_mode, int64_t ldo, void *workspace, size_t workspace_bytes, bwta_stream_t stream)
{
    if (count < 0) return BWTA_ERR_SHAPE;
    if (count == 0) return BWTA_OK;
    if (!problems) return BWTA_ERR_NULL;
    const size_t per = bwta_workspace_bytes(M, N, K);
    if (M > 0 && N > 0 && (!workspace || workspace_bytes < per * (size_t)count)) return BWTA_ERR_WORKSPACE;
    if (workspace && !aligned(workspace, 256)) return BWTA_ERR_ALIGN;
    for (int i = 0; i < count; ++i) {  // validate everything before enqueueing anything
        const bwta_gemm_problem &p = problems[i];
        int rc = check_gemm_common(M, N, K, p.s_a, p.s_a ? a_scale_mode : BWTA_SCALE_NONE, p.s_w,
                                   p.s_w ? w_scale_mode : BWTA_SCALE_NONE, p.out, ldo);
        if (rc != BWTA_OK) return rc;
        if (M == 0 || N == 0) continue;
        if (!p.mask || !p.sign || !p.wsign || (!p.acc && !p.out)) return BWTA_ERR_NULL;
        if (!aligned(p.mask, 16) || !aligned(p.sign, 16) || !aligned(p.wsign, 16)) return BWTA_ERR_ALIGN;
        if (p.acc && !aligned(p.acc, 4)) return BWTA_ERR_ALIGN;
    }
    if (M == 0 || N == 0) return BWTA_OK;
    hipStream_t st = (hipStream_t)stream;
    const int rw = (int)bwta_plane_row_words(K);
    auto args_of = [&](const bwta_gemm_problem &p) {
        return bwta::GemmArgs{p.mask, p.sign, p.wsign, M, N, K, rw,
                              {(const uint16_t *)p.s_a, p.s_a ? a_scale_mode : BWTA_SCALE_NONE},
                              {(const uint16_t *)p.s_w, p.s_w ? w_scale_mode : BWTA_SCALE_NONE},
                              p.acc, (uint16_t *)p.out, ldo};
    };
    bwta::GemmArgs first = args_of(problems[0]);
    const int path = resolve_path(M, N, K);
    const bool dec_fp4 = path == BWTA_PATH_FP4 && bwta::gemv_fp4_supported(first);
    if (dec_fp4 || (path == BWTA_PATH_POPC && bwta::gemv_popc_supported(first))) {
        bwta::GemmArgs batch[64];
        for (int base = 0; base < count; base += 64) {
            const int n = count - base < 64 ? count - base : 64;
            for (int i = 0; i < n; ++i) batch[i] = args_of(problems[base + i]);
            int rc = hip_result(dec_fp4 ? bwta::launch_gemv_fp4_grouped(batch, n, st)
                                        : bwta::launch_gemv_popc_grouped(batch, n, st));
            if (rc != BWTA_OK) return rc;
        }
        return BWTA_OK;
    }
    for (int i = 0; i < count; ++i) {
        int rc = run_gemm(args_of(problems[i]), (char *)workspace + per * (size_t)i, st);
        if (rc != BWTA_OK) return rc;
    }
    return BWTA_OK;
}

int bwta_quantize_pack_bool(const void *A, int64_t lda, const void *s_a, int scale_mode, int M, int K,
                            uint32_t *mask, bwta_stream_t stream)
{
    if (!scale_mode_ok(scale_mode)) return BWTA_ERR_UNSUPPORTED;
    if (M < 0 || K < 0 || (M > 0 && K == 0)) return BWTA_ERR_SHAPE;
    if (M == 0) return BWTA_OK;
    if (lda < K) return BWTA_ERR_SHAPE;
    if (!A || !mask) return BWTA_ERR_NULL;
    if (scale_mode != BWTA_SCALE_NONE && !s_a) return BWTA_ERR_NULL;
    if (!aligned(mask, 16) || !aligned(A, 2) || (s_a && !aligned(s_a, 2))) return BWTA_ERR_ALIGN;
    bwta::ScaleArg sa{(const uint16_t *)s_a, s_a ? scale_mode : BWTA_SCALE_NONE};
    return hip_result(bwta::launch_quantize_pack_bool(A, lda, sa, M, K, mask, (hipStream_t)stream));
}

int bwta_matmul_tt(const uint32_t *maskA, const uint32_t *signA, int64_t strideA, const uint32_t *maskB,
                   const uint32_t *signB, int64_t strideB, int batch, int M, int N, int K, const void *s_a,
                   int a_scale_mode, const void *s_b, int b_scale_mode, float alpha, int32_t *acc, void *out,
                   int64_t ldo, int64_t stride_out, bwta_stream_t stream)
{
    int rc = check_gemm_common(M, N, K, s_a, a_scale_mode, s_b, b_scale_mode, out, ldo);
    if (rc != BWTA_OK) return rc;
    if (batch < 0) return BWTA_ERR_SHAPE;
    if (batch == 0 || M == 0 || N == 0) return BWTA_OK;
    if (batch > 65535) return BWTA_ERR_UNSUPPORTED;  // grid.z
    if (!(alpha == alpha) || alpha - alpha != 0.0f) return BWTA_ERR_UNSUPPORTED;  // NaN / Inf
    if (!maskA || !maskB || (!acc && !out)) return BWTA_ERR_NULL;
    const int64_t rw = bwta_plane_row_words(K);
    if (batch > 1 && (strideA < (int64_t)M * rw || strideB < (int64_t)N * rw)) return BWTA_ERR_SHAPE;
    if (out && batch > 1 && stride_out < (int64_t)(M - 1) * ldo + N) return BWTA_ERR_SHAPE;
    if ((strideA & 3) || (strideB & 3)) return BWTA_ERR_ALIGN;  // batches keep the 16-byte alignment
    if (!aligned(maskA, 16) || !aligned(maskB, 16) || (signA && !aligned(signA, 16)) ||
        (signB && !aligned(signB, 16)) || (acc && !aligned(acc, 4)))
        return BWTA_ERR_ALIGN;
    bwta::MatmulTTArgs g{maskA, signA, maskB, signB, strideA, strideB, batch, M, N, K, (int)rw,
                         {(const uint16_t *)s_a, s_a ? a_scale_mode : BWTA_SCALE_NONE},
                         {(const uint16_t *)s_b, s_b ? b_scale_mode : BWTA_SCALE_NONE},
                         alpha, acc, (uint16_t *)out, ldo, (int64_t)M * N, stride_out};
    const bool popcount_kernel = g_path.load(std::memory_order_relaxed) == BWTA_PATH_POPC;  // comparison path
    return hip_result(bwta::launch_matmul_tt(g, popcount_kernel, (hipStream_t)stream));
}

int bwta_matmul_bool_prepared(const uint32_t *maskA, int64_t strideA, const void *preparedB, size_t preparedB_bytes,
                              int preparedB_format, int batch, int M, int N, int K, const void *s_a, int a_scale_mode, const void *s_b,
                              int b_scale_mode, float alpha, void *out, int64_t ldo, int64_t stride_out,
                              bwta_stream_t stream)
{
    int rc = check_gemm_common(M, N, K, s_a, a_scale_mode, s_b, b_scale_mode, out, ldo);
    if (rc != BWTA_OK) return rc;
    if (batch < 0) return BWTA_ERR_SHAPE;
    if (batch == 0 || M == 0 || N == 0) return BWTA_OK;
    if (batch > 65535) return BWTA_ERR_UNSUPPORTED;  // same limit as bwta_matmul_tt
    if (!(alpha == alpha) || alpha - alpha != 0.0f) return BWTA_ERR_UNSUPPORTED;  // NaN / Inf
    if (!maskA || !out) return BWTA_ERR_NULL;
    // a workgroup's tile takes 128 rows of B: batch entries must not share one.  The prepared operand
    // must hold matrix-core fragments, which bwta_prepare_act writes on the FP4 path above 128 rows.
    if ((N & 127) != 0 || (int64_t)batch * N > 0x7fffffff) return BWTA_ERR_UNSUPPORTED;
    const int rows_b = batch * N;
    if (preparedB_format != BWTA_PREPARED_FP4) return BWTA_ERR_UNSUPPORTED;
    const int64_t rw = bwta_plane_row_words(K);
    if (batch > 1 && strideA < (int64_t)M * rw) return BWTA_ERR_SHAPE;
    if (batch > 1 && stride_out < (int64_t)(M - 1) * ldo + N) return BWTA_ERR_SHAPE;
    if (strideA & 3) return BWTA_ERR_ALIGN;  // batches keep the 16-byte alignment
    if (!aligned(maskA, 16)) return BWTA_ERR_ALIGN;
    if (!preparedB || preparedB_bytes < bwta_prepared_bytes(rows_b, K)) return BWTA_ERR_WORKSPACE;
    if (!aligned(preparedB, 256)) return BWTA_ERR_ALIGN;
    const uint32_t *frag = (const uint32_t *)((const char *)preparedB + 2 * plane_bytes(rows_b, K));
    // in the tiled kernel's terms the fragment operand (B, N rows) is the "activation" side and the
    // boolean plane (A, M rows) the 1-bit "weight" side; its epilogue writes out[m][n]
    bwta::GemmArgs g{nullptr, nullptr, maskA, N, M, K, (int)rw,
                     {(const uint16_t *)s_b, s_b ? b_scale_mode : BWTA_SCALE_NONE},
                     {(const uint16_t *)s_a, s_a ? a_scale_mode : BWTA_SCALE_NONE},
                     nullptr, (uint16_t *)out, ldo};
    return hip_result(bwta::launch_att_v_fp4(g, frag, batch, strideA, stride_out, alpha, (hipStream_t)stream));
}

int bwta_prepare_weights(const void *W, int64_t ldw, int N, int K, uint32_t *wsign, void *s_w,
                         bwta_stream_t stream)
{
    if (N < 0 || K < 0 || (N > 0 && K == 0)) return BWTA_ERR_SHAPE;
    if (N == 0) return BWTA_OK;
    if (ldw < K) return BWTA_ERR_SHAPE;
    if (K > 32768) return BWTA_ERR_UNSUPPORTED;  // K * value must stay inside 64 bits
    if (!W || !wsign || !s_w) return BWTA_ERR_NULL;
    if (!aligned(wsign, 16) || !aligned(W, 2) || !aligned(s_w, 2)) return BWTA_ERR_ALIGN;
    return hip_result(bwta::launch_prepare_weights(W, ldw, N, K, wsign, (uint16_t *)s_w, (hipStream_t)stream));
}

int bwta_act_scale(const void *A, int64_t lda, int M, int K, void *s, bwta_stream_t stream)
{
    if (M < 0 || K < 0 || (M > 0 && K == 0)) return BWTA_ERR_SHAPE;
    if (M == 0) return BWTA_OK;
    if (lda < K) return BWTA_ERR_SHAPE;
    if (K > 32768) return BWTA_ERR_UNSUPPORTED;
    if (!A || !s) return BWTA_ERR_NULL;
    if (!aligned(A, 2) || !aligned(s, 2)) return BWTA_ERR_ALIGN;
    return hip_result(bwta::launch_act_scale(A, lda, M, K, (uint16_t *)s, (hipStream_t)stream));
}

const char *bwta_strerror(int code)
{
    switch (code) {
    case BWTA_OK: return "ok";
    case BWTA_ERR_NULL: return "a required pointer is NULL";
    case BWTA_ERR_SHAPE: return "invalid shape or leading dimension";
    case BWTA_ERR_ALIGN: return "misaligned pointer";
    case BWTA_ERR_UNSUPPORTED: return "unsupported dtype, scale mode or path";
    case BWTA_ERR_WORKSPACE: return "workspace missing or too small";
    case BWTA_ERR_HIP: return "HIP runtime error at launch (see bwta_last_hip_error)";
    case BWTA_ERR_TOO_LARGE: return "the shape needs more scratch than the library's static scratch holds";
    default: return "unknown error code";
    }
}

int bwta_last_hip_error(void) { return t_last_hip_error; }

int bwta_set_path(int path)
{
    if (path < BWTA_PATH_AUTO || path > BWTA_PATH_FP4) return BWTA_ERR_UNSUPPORTED;
    g_path.store(path, std::memory_order_relaxed);
    return BWTA_OK;
}

int bwta_get_path(void) { return g_path.load(std::memory_order_relaxed); }

int bwta_auto_path(int M, int N, int K)
{
    (void)N;
    (void)K;
    // one token: the popcount decode kernel; more: the FP4 matrix cores (decode kernel up to 128
    // tokens, tiled kernel above).  Measured: at two tokens the popcount kernel is level with the
    // matrix cores at K = 4096 and a third slower at K = 11008.
    return M > 1 ? BWTA_PATH_FP4 : BWTA_PATH_POPC;
}

int bwta_linear_launches(int M, int N, int K)
{
    if (M <= 0 || N <= 0 || K <= 0) return 0;
    if (resolve_path(M, N, K) != BWTA_PATH_FP4) return 2;
    alignas(16) static const uint16_t dense[8] = {};  // stands for an aligned input; never read
    uint16_t sink = 0;
    bwta::GemmArgs g{nullptr, nullptr, nullptr, M, N, K, (int)bwta_plane_row_words(K),
                     {nullptr, BWTA_SCALE_NONE}, {nullptr, BWTA_SCALE_NONE}, nullptr, &sink, N};
    return bwta::linear_fused_supported(dense, K, g) ? 1 : 2;
}

int bwta_planned_kernel(int operand, int M, int N, int K)
{
    if (M <= 0 || N <= 0 || K <= 0) return 0;
    if (operand == BWTA_PREPARED_FP4) return BWTA_KERNEL_GEMM_FP4;
    if (operand != 0 && operand != BWTA_PREPARED_PLANES) return 0;
    bwta::GemmArgs g{};
    g.M = M, g.N = N, g.K = K;
    g.rw = (int)bwta_plane_row_words(K);
    return plan_from_planes(g, operand == 0);
}

int bwta_version(void) { return 2; }

#ifndef BWTA_BUILD_ID
#define BWTA_BUILD_ID "unknown"
#endif
const char *bwta_build_id(void) { return BWTA_BUILD_ID; }

int bwta_set_tile(int tile)
{
    if (tile >= 2000) {  // matrix-core decode kernel: 2000 + 1024 * ring depth + 64 * chunks-per-wavefront + tiles-per-workgroup
        const int c = tile - 2000;
        bwta::set_gemv_fp4_tile((c / 64) % 16, c % 64, c / 1024);
        return BWTA_OK;
    }
    bwta::set_gemv_fp4_tile(0, 0, 0);
    if (tile >= 1000) {  // decode kernel: 1000 + 16 * lanes-per-row + chunks-per-lane
        bwta::set_gemv_tile((tile - 1000) / 16, (tile - 1000) % 16);
        return BWTA_OK;
    }
    bwta::set_gemv_tile(0, 0);
    if (tile >= 900 && tile < 1000) {  // one-launch linear: 900 never, 901 wherever it can run, 900 + R the same with R channel splits
        bwta::set_linear_fused(tile > 900 ? 2 : 0, tile > 901 ? tile - 900 : 0);
        return BWTA_OK;
    }
    bwta::set_linear_fused(1, 0);
    bwta::set_fp4_tile(tile);
    return BWTA_OK;
}

}  // extern "C"
