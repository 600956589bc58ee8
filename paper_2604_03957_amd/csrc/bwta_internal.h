// Internal declarations shared by the HIP translation units of libbwta.so.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bwta {

struct ScaleArg {
    const uint16_t *ptr;  // fp16 bits, device
    int mode;             // BWTA_SCALE_*
};

struct GemmArgs {
    const uint32_t *mask, *sign, *wsign;
    int M, N, K;
    int rw;  // words per packed row
    ScaleArg s_a, s_w;
    int32_t *acc;   // nullable
    uint16_t *out;  // nullable, fp16 bits
    int64_t ldo;
};

// launchers (each returns the launch's hipError_t)
hipError_t launch_quantize_pack(const void *A, int dtype, int64_t lda, ScaleArg s_a, int M, int K,
                                uint32_t *mask, uint32_t *sign, int32_t *nnz, hipStream_t st);
hipError_t launch_pack_weights(const void *W, int dtype, int64_t ldw, int N, int K, uint32_t *wsign,
                               hipStream_t st);
hipError_t launch_gemm_popc(const GemmArgs &g, hipStream_t st);
bool gemm_mfma_supported(const GemmArgs &g);
hipError_t launch_gemm_mfma(const GemmArgs &g, hipStream_t st);

// ---- device helpers -------------------------------------------------------------------------

__device__ __forceinline__ float half_bits_to_float(uint16_t h)
{
    _Float16 f;
    __builtin_memcpy(&f, &h, 2);
    return (float)f;
}

__device__ __forceinline__ float load_scale(const ScaleArg &s, int row)
{
    if (s.mode == 0 || s.ptr == nullptr) return 1.0f;
    return half_bits_to_float(s.ptr[s.mode == 1 ? 0 : row]);
}

// fp16( acc * s ) with a single rounding, where s = s_a * s_w is exact in fp32 (two 11-bit
// significands).  acc is exact in fp32 (|acc| < 2^24); the fp32 product is rounded to odd using
// the exact fma residual, so the final round-to-nearest-even to fp16 sees the true value.
__device__ __forceinline__ uint16_t scaled_to_half(int acc, float s)
{
    float a = (float)acc;
    float p = a * s;
    float e = __builtin_fmaf(a, s, -p);
    uint32_t b = __float_as_uint(p);
    if (e != 0.0f && __builtin_fabsf(p) < __builtin_inff()) {
        if ((e < 0.0f) != (p < 0.0f)) b -= 1u;  // true value lies towards zero from p
        b |= 1u;
    }
    const _Float16 r = (_Float16)__uint_as_float(b);  // v_cvt_f16_f32, round to nearest even
    uint16_t bits;
    __builtin_memcpy(&bits, &r, 2);
    return bits;
}

}  // namespace bwta
