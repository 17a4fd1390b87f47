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
    // When vecs is not NULL the input rows are not read from x: row b is the pairwise-dot
    // interaction of vecs[b] ([V][D] fp32, samples V*D floats apart) -- slot 0, then the strict lower
    // triangle of V V^T row by row -- computed by the block, zero-filled up to width[0].
    const float* vecs;
    int32_t V, D;
};
bool rec_fused_interact_ok(int32_t V, int32_t D);               // the fused kernel can take this interaction

// An offsets scan (lengths -> bag starts) that may ride along with another launch: the scan of
// a batch is a few blocks of latency-bound work, so it shares a launch with the dense stack's
// first fused run instead of standing alone in front of the pooling kernel.
struct rec_scan_job {
    const int32_t* lengths;
    int64_t n;              // number of bags
    int64_t* offsets;       // [n + 1]
};
int rec_scan_parallel_tiles(int64_t n);                          // > 0: independent tiles; 0: serial scan only
rec_status rec_scan_launch(const rec_scan_job& job, hipStream_t s);

// The interaction in front of a predictor stack: done inside the stack's first launch when that
// launch is a fused run and the shape allows, else by a launch of its own into out (row stride ldo,
// zero-filled up to zero_to), which must be the stack's x.
struct rec_interact_job {
    const float* vecs;      // [B][V][D]
    int32_t V, D;
    float* out;
    int64_t ldo;
    int32_t zero_to;
};

// `scan` (may be NULL): also run this scan in the same launch; it must have parallel tiles.
rec_status rec_fused_mlp_launch(const rec_fused_mlp_args& a, rec_dtype dt, const rec_scan_job* scan, hipStream_t s);

// rec_mlp_forward that also gets `scan` done no later than its first launch completes
// (inside that launch when it is a fused run, by a launch of its own otherwise).
rec_status rec_mlp_forward_scan(const void* const* W, const float* const* bias, const int32_t* widths, int32_t n_layers,
                                rec_dtype wdtype, rec_act hidden_act, rec_act final_act, const float* x, int64_t ldx,
                                float* y, int64_t ldy, int32_t B, void* workspace, size_t workspace_bytes, void* stream,
                                const rec_scan_job* scan, const rec_interact_job* inter = nullptr);

// rec_sls_forward in steps: all of it, only the argument checks, or only the pooling launch
// (the caller has enqueued the scan into rec_sls_workspace_offsets() on the same stream).
enum rec_sls_step { REC_SLS_ALL = 0, REC_SLS_CHECK_ONLY = 1, REC_SLS_POOL_ONLY = 2 };
rec_status rec_sls_forward_step(const float* const* tables, const int64_t* rows, int32_t T, int32_t D,
                                const int32_t* indices, int64_t n_indices, const int32_t* lengths, int32_t B, float* out,
                                int64_t out_stride_b, int64_t out_stride_t, void* workspace, size_t workspace_bytes,
                                void* stream, rec_sls_step step);
int64_t* rec_sls_workspace_offsets(void* workspace);

// rec_interact that also writes zeros into columns [D + V(V-1)/2, zero_to) of every output row
// (zero_to <= ldo): padding for a consumer whose k range is rounded up for alignment.
rec_status rec_interact_padded(const float* vecs, int32_t B, int32_t V, int32_t D, float* out, int64_t ldo,
                               int32_t zero_to, void* stream);

// ---- large bf16 layers (gemm_bf16.hip) --------------------------------------------------------
struct rec_gemm_plan {
    int bm, bn;     // output tile (rows x columns)
    int tiles;      // output tiles = blocks; 0: the kernel does not apply to this layer
};
rec_gemm_plan rec_gemm_bf16_plan(int M, int N, int K);
// Bytes of workspace one such layer needs (the bf16 copy of fp32 activations); grows with M.
size_t rec_gemm_bf16_workspace_bytes(int M, int N, int K, bool x_bf16);
// y = act(x W^T + bias); x fp32 (copied to bf16 first) or bf16.  `scan` (may be NULL, must have
// parallel tiles): run this offsets scan inside the layer's preparing launch.
rec_status rec_gemm_bf16_launch(const void* x, bool x_bf16, int64_t ldx, const void* W, const float* bias, void* y,
                                bool y_bf16, int64_t ldy, void* workspace, int M, int N, int K, int act,
                                const rec_scan_job* scan, hipStream_t s);
// The same for fp32 layers (K a multiple of 32, x and W 16-byte aligned, ldx a multiple of 4).
rec_gemm_plan rec_gemm_f32_plan(int M, int N, int K);
rec_status rec_gemm_f32_launch(const float* x, int64_t ldx, const float* W, const float* bias, float* y, int64_t ldy, int M,
                               int N, int K, int act, hipStream_t s);
