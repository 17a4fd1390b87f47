// Fully-connected stacks: y = act(x W^T + b), layer after layer.
//
// Section II-A ("Features", "Product Ranking") of the DeepRecSys paper: dense
// features pass through a stack of FC layers, and a predictor stack produces the
// click probability; Table I gives the widths.  Each layer is a dense
// contraction [B x n_in] . [n_out x n_in]^T, so it runs on the matrix cores:
// fp32 operands through v_mfma_f32_32x32x2_f32, bf16 operands (fp32 accumulate)
// through v_mfma_f32_32x32x16_bf16.  Both x and W are contiguous along the
// reduction dimension, so both are staged into LDS with the same row-major tile
// loader and read back as per-lane k-runs.
#include "rec_common.h"

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short ushort8 __attribute__((ext_vector_type(8)));
typedef unsigned short ushort4v __attribute__((ext_vector_type(4)));

constexpr int BM = 64, BN = 64;           // block tile; 4 waves as 2x2, each a 32x32 MFMA tile
constexpr int FC_THREADS = 256;

// MFMA 32x32 accumulator layout: register v of lane l holds
//   row = 8*(v/4) + 4*(l/32) + v%4,  col = l%32.
template <bool OUT_BF16>
__device__ __forceinline__ void fc_epilogue(const floatx16& acc, const float* __restrict__ bias, void* __restrict__ Cv,
                                            int64_t ldc, int M, int N, int row0, int col0, int lane, int act) {
    const int n = col0 + (lane & 31);
    if (n >= N) return;
    const float bv = bias[n];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int m = row0 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (m < M) {
            const float z = rec_apply_act(acc[v] + bv, act);
            if (OUT_BF16)
                static_cast<uint16_t*>(Cv)[(int64_t)m * ldc + n] = rec_f32_to_bf16_bits(z);
            else
                static_cast<float*>(Cv)[(int64_t)m * ldc + n] = z;
        }
    }
}

// ---------------------------------------------------------------- fp32 operands
constexpr int BK32 = 32;                  // k-extent of an LDS tile
constexpr int LD32 = BK32 + 4;            // padded row, keeps 16-byte alignment

// Stage a [64 x BK32] fp32 tile (rows r0.., columns k0..) of a row-major matrix into LDS,
// zero-filling outside [n_rows x K].
__device__ __forceinline__ void stage_f32(float (*dst)[LD32], const float* __restrict__ src, int64_t ld, int n_rows,
                                          int K, int r0, int k0, bool vec, int tid) {
#pragma unroll
    for (int i = 0; i < (BM * BK32 / 4) / FC_THREADS; ++i) {
        const int f = tid + i * FC_THREADS;
        const int r = f / (BK32 / 4), c = (f % (BK32 / 4)) * 4;
        const int gr = r0 + r, gk = k0 + c;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (gr < n_rows) {
            const float* p = src + (int64_t)gr * ld + gk;
            if (vec && gk + 3 < K) {
                v = *reinterpret_cast<const float4*>(p);
            } else {
                if (gk + 0 < K) v.x = p[0];
                if (gk + 1 < K) v.y = p[1];
                if (gk + 2 < K) v.z = p[2];
                if (gk + 3 < K) v.w = p[3];
            }
        }
        *reinterpret_cast<float4*>(&dst[r][c]) = v;
    }
}

__global__ __launch_bounds__(FC_THREADS) void fc_f32_kernel(const float* __restrict__ A, int64_t lda,
                                                            const float* __restrict__ W,
                                                            const float* __restrict__ bias, float* __restrict__ C,
                                                            int64_t ldc, int M, int N, int K, int act, int vec_a,
                                                            int vec_w) {
    __shared__ __attribute__((aligned(16))) float As[BM][LD32];
    __shared__ __attribute__((aligned(16))) float Ws[BN][LD32];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    floatx16 acc = {0};
    for (int k0 = 0; k0 < K; k0 += BK32) {
        stage_f32(As, A, lda, M, K, m0, k0, vec_a, tid);
        stage_f32(Ws, W, K, N, K, n0, k0, vec_w, tid);
        __syncthreads();
        // A lane owns 4 consecutive k of its row per step and feeds them to 4 MFMAs; x and W use
        // the same k assignment, so the sum over k is complete whatever the order.
#pragma unroll
        for (int kc = 0; kc < BK32 / 8; ++kc) {
            const float4 a = *reinterpret_cast<const float4*>(&As[wm * 32 + (lane & 31)][kc * 8 + (lane >> 5) * 4]);
            const float4 b = *reinterpret_cast<const float4*>(&Ws[wn * 32 + (lane & 31)][kc * 8 + (lane >> 5) * 4]);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b.z, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b.w, acc, 0, 0, 0);
        }
        __syncthreads();
    }
    fc_epilogue<false>(acc, bias, C, ldc, M, N, m0 + wm * 32, n0 + wn * 32, lane, act);
}

// ---------------------------------------------------------------- bf16 operands
constexpr int BK16 = 64;
constexpr int LD16 = BK16 + 8;            // padded row (in bf16 elements), keeps 16-byte alignment

// Stage a [64 x BK16] tile into LDS as bf16.  SRC_BF16: source already holds bf16 bit patterns;
// otherwise the source is fp32 and is rounded to nearest even here.
template <bool SRC_BF16>
__device__ __forceinline__ void stage_bf16(uint16_t (*dst)[LD16], const void* __restrict__ srcv, int64_t ld, int n_rows,
                                           int K, int r0, int k0, bool vec, int tid) {
    if (SRC_BF16) {
        const uint16_t* __restrict__ src = static_cast<const uint16_t*>(srcv);
#pragma unroll
        for (int i = 0; i < (BM * BK16 / 8) / FC_THREADS; ++i) {
            const int f = tid + i * FC_THREADS;
            const int r = f / (BK16 / 8), c = (f % (BK16 / 8)) * 8;
            const int gr = r0 + r, gk = k0 + c;
            ushort8 v = {0, 0, 0, 0, 0, 0, 0, 0};
            if (gr < n_rows) {
                const uint16_t* p = src + (int64_t)gr * ld + gk;
                if (vec && gk + 7 < K) {
                    v = *reinterpret_cast<const ushort8*>(p);
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (gk + e < K) v[e] = p[e];
                }
            }
            *reinterpret_cast<ushort8*>(&dst[r][c]) = v;
        }
    } else {
        const float* __restrict__ src = static_cast<const float*>(srcv);
#pragma unroll
        for (int i = 0; i < (BM * BK16 / 4) / FC_THREADS; ++i) {
            const int f = tid + i * FC_THREADS;
            const int r = f / (BK16 / 4), c = (f % (BK16 / 4)) * 4;
            const int gr = r0 + r, gk = k0 + c;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (gr < n_rows) {
                const float* p = src + (int64_t)gr * ld + gk;
                if (vec && gk + 3 < K) {
                    v = *reinterpret_cast<const float4*>(p);
                } else {
                    if (gk + 0 < K) v.x = p[0];
                    if (gk + 1 < K) v.y = p[1];
                    if (gk + 2 < K) v.z = p[2];
                    if (gk + 3 < K) v.w = p[3];
                }
            }
            ushort4v o = {rec_f32_to_bf16_bits(v.x), rec_f32_to_bf16_bits(v.y), rec_f32_to_bf16_bits(v.z),
                          rec_f32_to_bf16_bits(v.w)};
            *reinterpret_cast<ushort4v*>(&dst[r][c]) = o;
        }
    }
}

template <bool IN_BF16, bool OUT_BF16>
__global__ __launch_bounds__(FC_THREADS) void fc_bf16_kernel(const void* __restrict__ A, int64_t lda,
                                                             const uint16_t* __restrict__ W,
                                                             const float* __restrict__ bias, void* __restrict__ C,
                                                             int64_t ldc, int M, int N, int K, int act, int vec_a,
                                                             int vec_w) {
    __shared__ __attribute__((aligned(16))) uint16_t As[BM][LD16];
    __shared__ __attribute__((aligned(16))) uint16_t Ws[BN][LD16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    floatx16 acc = {0};
    for (int k0 = 0; k0 < K; k0 += BK16) {
        stage_bf16<IN_BF16>(As, A, lda, M, K, m0, k0, vec_a, tid);
        stage_bf16<true>(Ws, W, K, N, K, n0, k0, vec_w, tid);
        __syncthreads();
#pragma unroll
        for (int kc = 0; kc < BK16 / 16; ++kc) {
            const bf16x8 a = *reinterpret_cast<const bf16x8*>(&As[wm * 32 + (lane & 31)][kc * 16 + (lane >> 5) * 8]);
            const bf16x8 b = *reinterpret_cast<const bf16x8*>(&Ws[wn * 32 + (lane & 31)][kc * 16 + (lane >> 5) * 8]);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
        }
        __syncthreads();
    }
    fc_epilogue<OUT_BF16>(acc, bias, C, ldc, M, N, m0 + wm * 32, n0 + wn * 32, lane, act);
}

__global__ __launch_bounds__(256) void f32_to_bf16_kernel(const float* __restrict__ src, uint16_t* __restrict__ dst,
                                                          int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        dst[i] = rec_f32_to_bf16_bits(src[i]);
}

// Row stride (in elements) of an intermediate activation buffer of the given width.
int64_t hidden_ld(int32_t width, rec_dtype dt) {
    const int64_t q = (dt == REC_BF16) ? 8 : 4;
    return (width + q - 1) / q * q;
}

size_t hidden_buffer_bytes(const int32_t* widths, int32_t n_layers, int32_t B, rec_dtype dt) {
    int64_t mx = 0;
    for (int32_t l = 1; l < n_layers; ++l) mx = hidden_ld(widths[l], dt) > mx ? hidden_ld(widths[l], dt) : mx;
    return rec_round_up((size_t)mx * (size_t)B * (dt == REC_BF16 ? 2 : 4), 256);
}

rec_status launch_layer(const void* x, bool x_bf16, int64_t ldx, const void* W, rec_dtype dt, const float* bias,
                        int32_t B, int32_t n_in, int32_t n_out, int act, void* y, bool y_bf16, int64_t ldy,
                        hipStream_t s) {
    const dim3 grid((n_out + BN - 1) / BN, (B + BM - 1) / BM), block(FC_THREADS);
    if (dt == REC_F32) {
        const int vec_a = (ldx % 4 == 0) && rec_aligned(x, 16);
        const int vec_w = (n_in % 4 == 0) && rec_aligned(W, 16);
        hipLaunchKernelGGL(fc_f32_kernel, grid, block, 0, s, static_cast<const float*>(x), ldx,
                           static_cast<const float*>(W), bias, static_cast<float*>(y), ldy, B, n_out, n_in, act,
                           vec_a, vec_w);
    } else {
        const int vec_a = x_bf16 ? ((ldx % 8 == 0) && rec_aligned(x, 16)) : ((ldx % 4 == 0) && rec_aligned(x, 16));
        const int vec_w = (n_in % 8 == 0) && rec_aligned(W, 16);
        const uint16_t* Wb = static_cast<const uint16_t*>(W);
#define FC_BF16(IN, OUT)                                                                                       \
    hipLaunchKernelGGL((fc_bf16_kernel<IN, OUT>), grid, block, 0, s, x, ldx, Wb, bias, y, ldy, B, n_out, n_in, act, \
                       vec_a, vec_w)
        if (x_bf16 && y_bf16) FC_BF16(true, true);
        else if (x_bf16) FC_BF16(true, false);
        else if (y_bf16) FC_BF16(false, true);
        else FC_BF16(false, false);
#undef FC_BF16
    }
    REC_CHECK_LAUNCH();
    return REC_OK;
}

}  // namespace

extern "C" {

size_t rec_mlp_workspace_bytes(const int32_t* widths, int32_t n_layers, int32_t B, rec_dtype wdtype) {
    if (!widths || n_layers < 1 || B < 0) return 0;
    return 2 * hidden_buffer_bytes(widths, n_layers, B, wdtype);
}

rec_status rec_mlp_forward(const void* const* W, const float* const* bias, const int32_t* widths,
                           int32_t n_layers, rec_dtype wdtype, rec_act hidden_act, rec_act final_act,
                           const float* x, int64_t ldx, float* y, int64_t ldy, int32_t B, void* workspace,
                           size_t workspace_bytes, void* stream) {
    if (!W || !bias || !widths) return REC_ERR_NULL;
    if (n_layers < 1 || B < 0) return REC_ERR_BAD_SHAPE;
    if (wdtype != REC_F32 && wdtype != REC_BF16) return REC_ERR_UNSUPPORTED;
    if ((int)hidden_act < 0 || (int)hidden_act > 2 || (int)final_act < 0 || (int)final_act > 2)
        return REC_ERR_UNSUPPORTED;
    for (int32_t l = 0; l <= n_layers; ++l)
        if (widths[l] < 1) return REC_ERR_BAD_SHAPE;
    for (int32_t l = 0; l < n_layers; ++l)
        if (!W[l] || !bias[l]) return REC_ERR_NULL;
    if (B == 0) return REC_OK;
    if (!x || !y) return REC_ERR_NULL;
    if (ldx < widths[0] || ldy < widths[n_layers]) return REC_ERR_BAD_SHAPE;
    const size_t half = hidden_buffer_bytes(widths, n_layers, B, wdtype);
    if (n_layers > 1 && (!workspace || !rec_aligned(workspace, 256) || workspace_bytes < 2 * half))
        return REC_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool bf = (wdtype == REC_BF16);
    const void* cur = x;
    int64_t ld = ldx;
    bool cur_bf16 = false;
    for (int32_t l = 0; l < n_layers; ++l) {
        const bool last = (l == n_layers - 1);
        void* dst = last ? static_cast<void*>(y) : static_cast<void*>(static_cast<char*>(workspace) + (l & 1) * half);
        const int64_t ldd = last ? ldy : hidden_ld(widths[l + 1], wdtype);
        rec_status st = launch_layer(cur, cur_bf16, ld, W[l], wdtype, bias[l], B, widths[l], widths[l + 1],
                                     last ? (int)final_act : (int)hidden_act, dst, bf && !last, ldd, s);
        if (st != REC_OK) return st;
        cur = dst;
        ld = ldd;
        cur_bf16 = bf && !last;
    }
    return REC_OK;
}

rec_status rec_f32_to_bf16(const float* src, uint16_t* dst, int64_t n, void* stream) {
    if (n < 0) return REC_ERR_BAD_SHAPE;
    if (n == 0) return REC_OK;
    if (!src || !dst) return REC_ERR_NULL;
    const int64_t blocks = (n + 255) / 256;
    hipLaunchKernelGGL(f32_to_bf16_kernel, dim3((unsigned)(blocks < 4096 ? blocks : 4096)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), src, dst, n);
    REC_CHECK_LAUNCH();
    return REC_OK;
}

}  // extern "C"
