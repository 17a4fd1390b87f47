// Fully-connected stacks: y = act(x W^T + b), layer after layer.
//
// Section II-A ("Features", "Product Ranking") of the DeepRecSys paper: dense
// features pass through a stack of FC layers, and a predictor stack produces the
// click probability; Table I gives the widths.  Each layer is a dense
// contraction [B x n_in] . [n_out x n_in]^T, so it runs on the matrix cores:
// fp32 operands through v_mfma_f32_32x32x2_f32, bf16 operands (fp32 accumulate)
// through v_mfma_f32_32x32x16_bf16.
//
// The layers of these models are small (a batch of a few hundred to a thousand
// rows, widths 1..1024), so the kernel is built to fill 256 CUs from little
// work: a block owns a (32*WM) x (32*WN) output tile and KS groups of waves
// split the reduction dimension between them (in-block split-K, folded through
// LDS in a fixed order, so results are reproducible).  x and W are both
// contiguous along k and go through the same row-major tile loader into
// double-buffered LDS; the next tile's global loads are in flight while the
// current tile is multiplied.
#include "rec_common.h"

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short ushort8 __attribute__((ext_vector_type(8)));
typedef unsigned short ushort4v __attribute__((ext_vector_type(4)));

template <int WM_, int WN_, int KS_, bool BF16_>
struct FcCfg {
    static constexpr int WM = WM_, WN = WN_, KS = KS_;
    static constexpr bool BF16 = BF16_;
    static constexpr int BM = 32 * WM, BN = 32 * WN;
    static constexpr int WAVES = WM * WN * KS;
    static constexpr int THREADS = 64 * WAVES;
    // k-extent one wave consumes per tile, and k-extent of the whole staged tile
    static constexpr int BKW = BF16 ? (KS == 1 ? 64 : (KS == 8 ? 16 : 32)) : (KS == 1 ? 32 : (KS == 8 ? 8 : 16));
    static constexpr int KT = BKW * KS;
    static constexpr int ELT = BF16 ? 2 : 4;                  // bytes per LDS element
    static constexpr int LD = KT + 16 / ELT;                  // padded LDS row (elements), 16-byte multiple
    static constexpr int TILE_BYTES = (BM + BN) * LD * ELT;   // one stage: x tile then W tile
    static constexpr int RED_BYTES = (KS - 1) * WM * WN * 16 * 64 * 4;
    static constexpr int LDS_BYTES = (2 * TILE_BYTES > RED_BYTES) ? 2 * TILE_BYTES : RED_BYTES;
    static constexpr int STAGES = (WAVES >= 16) ? 3 : 4;                          // tiles of global loads in flight
};

// ---- global -> register -> LDS staging of a [ROWS x KT] tile -----------------------------------
// MODE 0: fp32 source -> fp32 LDS;  MODE 1: fp32 source -> bf16 LDS (rounded to nearest even here);
// MODE 2: bf16 source -> bf16 LDS.  A thread moves PER vectors of VEC source elements.
template <int MODE, int ROWS, int KT, int THREADS>
struct Stage {
    static constexpr int VEC = (MODE == 2) ? 8 : 4;
    static constexpr int UNITS = ROWS * KT / VEC;
    static constexpr int PER = (UNITS + THREADS - 1) / THREADS;
    static constexpr bool EXACT = (UNITS % THREADS == 0);
    typedef typename std::conditional<MODE == 2, ushort8, float4>::type reg_t;
    typedef typename std::conditional<MODE == 2, uint16_t, float>::type src_t;
    typedef typename std::conditional<MODE == 0, float, uint16_t>::type lds_t;
    reg_t r[PER];

    __device__ __forceinline__ void load(const void* __restrict__ srcv, int64_t ld, int n_rows, int K, int r0, int k0,
                                         bool vec, int tid) {
        const src_t* __restrict__ src = static_cast<const src_t*>(srcv);
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int f = tid + i * THREADS;
            const int row = f / (KT / VEC), c = (f % (KT / VEC)) * VEC;
            const int gr = r0 + row, gk = k0 + c;
            reg_t v;
            if constexpr (MODE == 2) v = reg_t{0, 0, 0, 0, 0, 0, 0, 0};
            else v = make_float4(0.f, 0.f, 0.f, 0.f);
            if ((EXACT || f < UNITS) && gr < n_rows && gk < K) {
                const src_t* p = src + (int64_t)gr * ld + gk;
                if (vec && gk + VEC - 1 < K) {
                    v = *reinterpret_cast<const reg_t*>(p);
                } else if constexpr (MODE == 2) {
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (gk + e < K) v[e] = p[e];
                } else {
                    v.x = p[0];
                    if (gk + 1 < K) v.y = p[1];
                    if (gk + 2 < K) v.z = p[2];
                    if (gk + 3 < K) v.w = p[3];
                }
            }
            r[i] = v;
        }
    }
    __device__ __forceinline__ void store(void* dstv, int ldl, int tid) const {
        lds_t* dst = static_cast<lds_t*>(dstv);
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int f = tid + i * THREADS;
            const int row = f / (KT / VEC), c = (f % (KT / VEC)) * VEC;
            if (EXACT || f < UNITS) {
                if constexpr (MODE == 1) {
                    const ushort4v o = {rec_f32_to_bf16_bits(r[i].x), rec_f32_to_bf16_bits(r[i].y),
                                        rec_f32_to_bf16_bits(r[i].z), rec_f32_to_bf16_bits(r[i].w)};
                    *reinterpret_cast<ushort4v*>(dst + row * ldl + c) = o;
                } else {
                    *reinterpret_cast<reg_t*>(dst + row * ldl + c) = r[i];
                }
            }
        }
    }
};

// MFMA 32x32 accumulator layout: register v of lane l holds
//   row = 8*(v/4) + 4*(l/32) + v%4,  col = l%32.
__device__ __forceinline__ void fc_epilogue(const floatx16& acc, const float* __restrict__ bias, void* __restrict__ Cv,
                                            bool c_bf16, int64_t ldc, int M, int N, int row0, int col0, int lane,
                                            int act) {
    const int n = col0 + (lane & 31);
    if (n >= N) return;
    const float bv = bias[n];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int m = row0 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (m < M) {
            const float z = rec_apply_act(acc[v] + bv, act);
            if (c_bf16)
                static_cast<uint16_t*>(Cv)[(int64_t)m * ldc + n] = rec_f32_to_bf16_bits(z);
            else
                static_cast<float*>(Cv)[(int64_t)m * ldc + n] = z;
        }
    }
}

// C[M x N] = act(A[M x K] . W[N x K]^T + bias).
//   fp32 mode: A, W fp32.   bf16 mode: W bf16; A fp32 (A_BF16 = false, rounded while staged) or bf16.
//   C fp32, or bf16 (bf16 mode, hidden layers: the rounding the next layer's operand needs anyway).
// Global loads run STAGES tiles ahead of the multiply (held in registers until their LDS slot is
// free), so several tiles' worth of latency is covered per block.
template <class Cfg, bool A_BF16>
__global__ __launch_bounds__(Cfg::THREADS) void fc_kernel(const void* __restrict__ A, int64_t lda,
                                                          const void* __restrict__ W, const float* __restrict__ bias,
                                                          void* __restrict__ C, int c_bf16, int64_t ldc, int M, int N,
                                                          int K, int act, int vec_a, int vec_w) {
    constexpr int BM = Cfg::BM, BN = Cfg::BN, KT = Cfg::KT, LD = Cfg::LD, BKW = Cfg::BKW, THREADS = Cfg::THREADS;
    constexpr int P = Cfg::STAGES;
    constexpr int ELT = Cfg::ELT;
    constexpr int MODE_A = Cfg::BF16 ? (A_BF16 ? 2 : 1) : 0;
    constexpr int MODE_W = Cfg::BF16 ? 2 : 0;
    __shared__ __attribute__((aligned(16))) unsigned char lds[Cfg::LDS_BYTES];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % Cfg::WM, wn = (wave / Cfg::WM) % Cfg::WN, ks = wave / (Cfg::WM * Cfg::WN);
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int n_tiles = (K + KT - 1) / KT;
    floatx16 acc = {0};

    Stage<MODE_A, BM, KT, THREADS> sa[P];
    Stage<MODE_W, BN, KT, THREADS> sw[P];
    auto tileA = [&](int s) { return lds + s * Cfg::TILE_BYTES; };
    auto tileW = [&](int s) { return lds + s * Cfg::TILE_BYTES + BM * LD * ELT; };

#pragma unroll
    for (int p = 0; p < P; ++p) {
        if (p < n_tiles) {
            sa[p].load(A, lda, M, K, m0, p * KT, vec_a, tid);
            sw[p].load(W, K, N, K, n0, p * KT, vec_w, tid);
        }
    }
    sa[0].store(tileA(0), LD, tid);
    sw[0].store(tileW(0), LD, tid);
    __syncthreads();

    const int lds_off = ((lane & 31)) * LD + ks * BKW + (lane >> 5) * (Cfg::BF16 ? 8 : 4);
    for (int it0 = 0; it0 < n_tiles; it0 += P) {
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const int it = it0 + p;
            if (it < n_tiles) {
                const int cur = it & 1;
                if (it + P < n_tiles) {      // stage p was written to LDS one step ago: refill it
                    sa[p].load(A, lda, M, K, m0, (it + P) * KT, vec_a, tid);
                    sw[p].load(W, K, N, K, n0, (it + P) * KT, vec_w, tid);
                }
                if constexpr (!Cfg::BF16) {
                    // A lane owns 4 consecutive k of its row per step and feeds them to 4 MFMAs; x and W
                    // use the same k assignment, so the sum over k is complete whatever the order.
                    const float* pa = reinterpret_cast<const float*>(tileA(cur)) + wm * 32 * LD + lds_off;
                    const float* pw = reinterpret_cast<const float*>(tileW(cur)) + wn * 32 * LD + lds_off;
#pragma unroll
                    for (int kc = 0; kc < BKW / 8; ++kc) {
                        const float4 a = *reinterpret_cast<const float4*>(pa + kc * 8);
                        const float4 b = *reinterpret_cast<const float4*>(pw + kc * 8);
                        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, acc, 0, 0, 0);
                        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, acc, 0, 0, 0);
                        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b.z, acc, 0, 0, 0);
                        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b.w, acc, 0, 0, 0);
                    }
                } else {
                    const uint16_t* pa = reinterpret_cast<const uint16_t*>(tileA(cur)) + wm * 32 * LD + lds_off;
                    const uint16_t* pw = reinterpret_cast<const uint16_t*>(tileW(cur)) + wn * 32 * LD + lds_off;
#pragma unroll
                    for (int kc = 0; kc < BKW / 16; ++kc) {
                        const bf16x8 a = *reinterpret_cast<const bf16x8*>(pa + kc * 16);
                        const bf16x8 b = *reinterpret_cast<const bf16x8*>(pw + kc * 16);
                        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
                    }
                }
                if (it + 1 < n_tiles) {
                    sa[(p + 1) % P].store(tileA(cur ^ 1), LD, tid);
                    sw[(p + 1) % P].store(tileW(cur ^ 1), LD, tid);
                }
                __syncthreads();
            }
        }
    }

    // fold the KS partial tiles in the fixed order ks = 1, 2, ... (the loop above ended on a barrier,
    // so the staging buffers are free to be reused)
    if constexpr (Cfg::KS > 1) {
        float* red = reinterpret_cast<float*>(lds);
        const int tile_slot = (wn * Cfg::WM + wm) * 16 * 64;
        if (ks > 0) {
            float* dst = red + (ks - 1) * Cfg::WM * Cfg::WN * 16 * 64 + tile_slot;
#pragma unroll
            for (int v = 0; v < 16; ++v) dst[v * 64 + lane] = acc[v];
        }
        __syncthreads();
        if (ks > 0) return;
#pragma unroll
        for (int s = 1; s < Cfg::KS; ++s) {
            const float* src = red + (s - 1) * Cfg::WM * Cfg::WN * 16 * 64 + tile_slot;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] += src[v * 64 + lane];
        }
    }
    fc_epilogue(acc, bias, C, c_bf16 != 0, ldc, M, N, m0 + wm * 32, n0 + wn * 32, lane, act);
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

// A layer is "narrow" when 16 rows of its input and output fit the fused kernel's LDS buffers and
// its weights are small enough for every block to stream them from L2 (about half a MB).
bool layer_is_narrow(int32_t n_in, int32_t n_out, bool bf16) {
    const int32_t maxw = bf16 ? REC_FUSED_MAX_WIDTH_BF16 : REC_FUSED_MAX_WIDTH_F32;
    return n_in <= maxw && n_out <= maxw && (int64_t)n_in * n_out <= 128 * 1024;
}

template <class Cfg>
void launch_cfg(const void* x, int x_bf16, int64_t ldx, const void* W, const float* bias, void* y, int y_bf16,
                int64_t ldy, int M, int N, int K, int act, int vec_a, int vec_w, hipStream_t s) {
    const dim3 grid((N + Cfg::BN - 1) / Cfg::BN, (M + Cfg::BM - 1) / Cfg::BM), block(Cfg::THREADS);
    if (Cfg::BF16 && x_bf16)
        hipLaunchKernelGGL((fc_kernel<Cfg, Cfg::BF16>), grid, block, 0, s, x, ldx, W, bias, y, y_bf16, ldy, M, N, K,
                           act, vec_a, vec_w);
    else
        hipLaunchKernelGGL((fc_kernel<Cfg, false>), grid, block, 0, s, x, ldx, W, bias, y, y_bf16, ldy, M, N, K, act,
                           vec_a, vec_w);
}

template <bool BF16>
void launch_dtype(int shape, int ksplit, const void* x, int x_bf16, int64_t ldx, const void* W, const float* bias,
                  void* y, int y_bf16, int64_t ldy, int M, int N, int K, int act, int vec_a, int vec_w,
                  hipStream_t s) {
#define FC_GO(WM, WN, KS) \
    launch_cfg<FcCfg<WM, WN, KS, BF16>>(x, x_bf16, ldx, W, bias, y, y_bf16, ldy, M, N, K, act, vec_a, vec_w, s)
    if (shape == 2) {
        if (ksplit >= 4) FC_GO(2, 2, 4);
        else if (ksplit == 2) FC_GO(2, 2, 2);
        else FC_GO(2, 2, 1);
    } else if (shape == 1) {
        if (ksplit >= 8) FC_GO(2, 1, 8);
        else if (ksplit == 4) FC_GO(2, 1, 4);
        else if (ksplit == 2) FC_GO(2, 1, 2);
        else FC_GO(2, 1, 1);
    } else {
        if (ksplit >= 8) FC_GO(1, 1, 8);
        else if (ksplit == 4) FC_GO(1, 1, 4);
        else if (ksplit == 2) FC_GO(1, 1, 2);
        else FC_GO(1, 1, 1);
    }
#undef FC_GO
}

// Tile shape and in-block split-K for one layer.  Larger tiles reuse each staged operand more,
// but these layers are small: take the largest tile (64x64, 64x32, 32x32) that still gives the
// 256 CUs about a block each, then split k until there are about two waves per SIMD, as long as
// every k-group keeps a few steps of work.
void choose_shape(int M, int N, int K, bool bf16, int* shape, int* ksplit) {
    const int64_t t64 = (int64_t)((M + 63) / 64) * ((N + 63) / 64);
    const int64_t t6432 = (int64_t)((M + 63) / 64) * ((N + 31) / 32);
    const int64_t t32 = (int64_t)((M + 31) / 32) * ((N + 31) / 32);
    int64_t waves;
    int max_ks;
    if (t64 >= 200) { *shape = 2; waves = t64 * 4; max_ks = 4; }
    else if (t6432 >= 200) { *shape = 1; waves = t6432 * 2; max_ks = 8; }
    else { *shape = 0; waves = t32; max_ks = 8; }
    const int min_k = bf16 ? 64 : 32;
    int ks = 1;
    while (ks < max_ks && waves * ks < 2048 && K / (ks * 2) >= min_k) ks *= 2;
    *ksplit = ks;
}

// Bytes the layers that take the large-tile bf16 kernel need beyond the activation buffers (they run
// one after another and share the area).  Reserved for the first layer whatever kernel a given batch
// size ends up on, so the total never shrinks as B grows.
size_t gemm_area_bytes(const int32_t* widths, int32_t n_layers, int32_t B, rec_dtype dt) {
    size_t mx = 0;
    if (dt != REC_BF16) return 0;
    if (widths[0] % 64 == 0 && widths[0] >= 256) mx = rec_gemm_bf16_workspace_bytes(B, widths[1], widths[0], false);
    (void)n_layers;
    return mx;
}

// The large-tile bf16 kernel takes this layer: big enough, aligned for 16-byte loads.
bool layer_takes_gemm(const void* x, bool x_bf16, int64_t ldx, const void* W, rec_dtype dt, int32_t B, int32_t n_in,
                      int32_t n_out) {
    return dt == REC_BF16 && rec_gemm_bf16_plan(B, n_out, n_in).tiles != 0 && rec_aligned(x, 16) && rec_aligned(W, 16) &&
           ldx % (x_bf16 ? 8 : 4) == 0 && (!x_bf16 || (int64_t)B * ldx * 2 < ((int64_t)1 << 32));
}

rec_status launch_layer(const void* x, bool x_bf16, int64_t ldx, const void* W, rec_dtype dt, const float* bias,
                        int32_t B, int32_t n_in, int32_t n_out, int act, void* y, bool y_bf16, int64_t ldy,
                        void* gemm_area, const rec_scan_job* scan, hipStream_t s) {
    if (layer_takes_gemm(x, x_bf16, ldx, W, dt, B, n_in, n_out))
        return rec_gemm_bf16_launch(x, x_bf16, ldx, W, bias, y, y_bf16, ldy, gemm_area, B, n_out, n_in, act, scan, s);
    if (dt == REC_F32 && rec_gemm_f32_plan(B, n_out, n_in).tiles != 0 && rec_aligned(x, 16) && rec_aligned(W, 16) &&
        ldx % 4 == 0 && (int64_t)B * ldx * 4 < ((int64_t)1 << 32))
        return rec_gemm_f32_launch(static_cast<const float*>(x), ldx, static_cast<const float*>(W), bias, static_cast<float*>(y),
                                   ldy, B, n_out, n_in, act, s);
    int shape, ksplit;
    choose_shape(B, n_out, n_in, dt == REC_BF16, &shape, &ksplit);
    if (dt == REC_F32) {
        const int vec_a = (ldx % 4 == 0) && rec_aligned(x, 16);
        const int vec_w = (n_in % 4 == 0) && rec_aligned(W, 16);
        launch_dtype<false>(shape, ksplit, x, 0, ldx, W, bias, y, 0, ldy, B, n_out, n_in, act, vec_a, vec_w, s);
    } else {
        const int vec_a = x_bf16 ? ((ldx % 8 == 0) && rec_aligned(x, 16)) : ((ldx % 4 == 0) && rec_aligned(x, 16));
        const int vec_w = (n_in % 8 == 0) && rec_aligned(W, 16);
        launch_dtype<true>(shape, ksplit, x, x_bf16, ldx, W, bias, y, y_bf16, ldy, B, n_out, n_in, act, vec_a, vec_w, s);
    }
    REC_CHECK_LAUNCH();
    return REC_OK;
}

}  // namespace

extern "C" {

size_t rec_mlp_workspace_bytes(const int32_t* widths, int32_t n_layers, int32_t B, rec_dtype wdtype) {
    if (!widths || n_layers < 1 || B < 0) return 0;
    for (int32_t l = 0; l <= n_layers; ++l)
        if (widths[l] < 1) return 0;
    return 2 * hidden_buffer_bytes(widths, n_layers, B, wdtype) + gemm_area_bytes(widths, n_layers, B, wdtype);
}

rec_status rec_mlp_forward(const void* const* W, const float* const* bias, const int32_t* widths,
                           int32_t n_layers, rec_dtype wdtype, rec_act hidden_act, rec_act final_act,
                           const float* x, int64_t ldx, float* y, int64_t ldy, int32_t B, void* workspace,
                           size_t workspace_bytes, void* stream) {
    return rec_mlp_forward_scan(W, bias, widths, n_layers, wdtype, hidden_act, final_act, x, ldx, y, ldy, B, workspace,
                                workspace_bytes, stream, nullptr);
}

}  // extern "C"

rec_status rec_mlp_forward_scan(const void* const* W, const float* const* bias, const int32_t* widths, int32_t n_layers,
                                rec_dtype wdtype, rec_act hidden_act, rec_act final_act, const float* x, int64_t ldx,
                                float* y, int64_t ldy, int32_t B, void* workspace, size_t workspace_bytes, void* stream,
                                const rec_scan_job* scan, const rec_interact_job* inter) {
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
    const size_t need = 2 * half + gemm_area_bytes(widths, n_layers, B, wdtype);
    if (need > 0 && (!workspace || !rec_aligned(workspace, 256) || workspace_bytes < need)) return REC_ERR_WORKSPACE;
    void* gemm_area = static_cast<char*>(workspace) + 2 * half;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool bf = (wdtype == REC_BF16);
    const void* cur = x;
    int64_t ld = ldx;
    bool cur_bf16 = false;
    int32_t l = 0;
    int n_launch = 0;                 // alternates the two workspace halves
    // a run of narrow layers goes through the fused kernel, anything else through the tiled one
    auto narrow_run = [&](int32_t from) {
        int32_t run = 0;
        while (from + run < n_layers && run < REC_FUSED_MAX_LAYERS &&
               layer_is_narrow(widths[from + run], widths[from + run + 1], bf))
            ++run;
        return run;
    };
    if (scan) {
        // the scan rides in the stack's first launch that can carry it -- a fused run of narrow layers,
        // or the preparing launch of a large-tile layer; without one (or when the scan has no parallel
        // tiles) it gets a launch of its own up front
        bool can_ride = false;
        {
            bool in_bf16 = false;
            int64_t in_ld = ldx;
            const void* in = x;
            for (int32_t i = 0; i < n_layers && !can_ride;) {
                const int32_t run = narrow_run(i);
                can_ride = run > 0 || layer_takes_gemm(in, in_bf16, in_ld, W[i], wdtype, B, widths[i], widths[i + 1]);
                i += run > 0 ? run : 1;
                in = workspace;                       // hidden activations: 256-byte aligned halves of the workspace
                in_bf16 = bf;
                in_ld = hidden_ld(widths[i < n_layers ? i : n_layers], wdtype);
            }
        }
        if (!can_ride || rec_scan_parallel_tiles(scan->n) < 1) {
            const rec_status st = rec_scan_launch(*scan, s);
            if (st != REC_OK) return st;
            scan = nullptr;
        }
    }
    if (inter) {
        // the interaction is computed by the first launch when that is a fused run that can take it,
        // else by its own kernel into the stack's input buffer
        if (inter->out != x || inter->ldo != ldx) return REC_ERR_BAD_SHAPE;
        if (!(narrow_run(0) > 0 && rec_fused_interact_ok(inter->V, inter->D))) {
            const rec_status st = rec_interact_padded(inter->vecs, B, inter->V, inter->D, inter->out, inter->ldo, inter->zero_to,
                                                      stream);
            if (st != REC_OK) return st;
            inter = nullptr;
        }
    }
    while (l < n_layers) {
        const int32_t run = narrow_run(l);
        const int32_t l_end = run > 0 ? l + run : l + 1;
        const bool last = (l_end == n_layers);
        void* dst = last ? static_cast<void*>(y)
                         : static_cast<void*>(static_cast<char*>(workspace) + (n_launch & 1) * half);
        const int64_t ldd = last ? ldy : hidden_ld(widths[l_end], wdtype);
        rec_status st;
        if (run > 0) {
            rec_fused_mlp_args a;
            for (int32_t i = 0; i < run; ++i) {
                a.W[i] = W[l + i];
                a.bias[i] = bias[l + i];
                a.width[i] = widths[l + i];
                a.act[i] = (l + i == n_layers - 1) ? (int)final_act : (int)hidden_act;
            }
            a.width[run] = widths[l_end];
            a.n_layers = run;
            a.x = cur;
            a.x_bf16 = cur_bf16;
            a.ldx = ld;
            a.y = dst;
            a.y_bf16 = bf && !last;
            a.ldy = ldd;
            a.B = B;
            a.vecs = (l == 0 && inter) ? inter->vecs : nullptr;
            a.V = inter ? inter->V : 0;
            a.D = inter ? inter->D : 0;
            st = rec_fused_mlp_launch(a, wdtype, scan, s);
            scan = nullptr;
        } else {
            const bool carries = scan && layer_takes_gemm(cur, cur_bf16, ld, W[l], wdtype, B, widths[l], widths[l + 1]);
            st = launch_layer(cur, cur_bf16, ld, W[l], wdtype, bias[l], B, widths[l], widths[l + 1],
                              last ? (int)final_act : (int)hidden_act, dst, bf && !last, ldd, gemm_area,
                              carries ? scan : nullptr, s);
            if (carries) scan = nullptr;
        }
        if (st != REC_OK) return st;
        cur = dst;
        ld = ldd;
        cur_bf16 = bf && !last;
        l = l_end;
        ++n_launch;
    }
    return REC_OK;
}

extern "C" {

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
