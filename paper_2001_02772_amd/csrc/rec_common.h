// Internal helpers shared by the librec translation units (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "rec.h"

#define REC_WAVE 64

#define REC_CHECK_LAUNCH()                                   \
    do {                                                     \
        if (hipGetLastError() != hipSuccess) return REC_ERR_DEVICE; \
    } while (0)

static inline bool rec_aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
static inline size_t rec_round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// fp32 -> bf16 bit pattern, round to nearest even; NaN stays a (quiet) NaN.
__device__ __forceinline__ uint16_t rec_f32_to_bf16_bits(float x) {
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float rec_apply_act(float z, int act) {
    if (act == REC_ACT_RELU) return z > 0.0f ? z : 0.0f;
    if (act == REC_ACT_SIGMOID) return 1.0f / (1.0f + expf(-z));
    return z;
}

__device__ __forceinline__ bool rec_dev_aligned(const void* p, size_t a) {
    return (reinterpret_cast<uintptr_t>(p) % a) == 0;
}

// ---- several narrow FC layers in one launch (fc_fused.hip) ----------------------------------
#define REC_FUSED_MAX_LAYERS 4
#define REC_FUSED_MAX_WIDTH_F32 512      // widest activation row kept in LDS, fp32 stacks
#define REC_FUSED_MAX_WIDTH_BF16 1024    // ... and bf16 stacks

struct rec_fused_mlp_args {
    const void* W[REC_FUSED_MAX_LAYERS];      // [width[l+1]][width[l]] row-major, fp32 or bf16 patterns
    const float* bias[REC_FUSED_MAX_LAYERS];
    int32_t width[REC_FUSED_MAX_LAYERS + 1];
    int32_t act[REC_FUSED_MAX_LAYERS];
    int32_t n_layers;
    const void* x;                            // fp32, or bf16 patterns when x_bf16 (bf16 stacks only)
    int32_t x_bf16;
    int64_t ldx;
    void* y;                                  // fp32, or bf16 patterns when y_bf16
    int32_t y_bf16;
    int64_t ldy;
    int32_t B;
};

rec_status rec_fused_mlp_launch(const rec_fused_mlp_args& a, rec_dtype dt, hipStream_t s);

// ---- large bf16 layers (gemm_bf16.hip) --------------------------------------------------------
int rec_gemm_bf16_split(int M, int N, int K);                    // 0: kernel does not apply
size_t rec_gemm_bf16_partial_bytes(int M, int N, int K);         // fp32 partial tiles for the k split
rec_status rec_gemm_bf16_launch(const void* x, bool x_bf16, int64_t ldx, const void* W, const float* bias, void* y,
                                bool y_bf16, int64_t ldy, float* partial, int M, int N, int K, int act,
                                hipStream_t s);
