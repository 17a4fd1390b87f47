// Large bf16 FC layers: C = act(A W^T + b) with A [M x K], W [N x K] bf16, fp32 accumulate.
//
// This is the one genuinely dense, FLOP-heavy contraction of the models in Table I of the
// DeepRecSys paper: the first Dense-FC layer of the MLP-dominated DLRM-RMC3 (thousands of dense
// inputs into a 1024-wide layer; Section III-A: its run time is dominated by FC layers).
// 128x128 output tile per block, four waves each owning a 64x64 quarter as 2x2
// v_mfma_f32_32x32x16_bf16 tiles, k staged 64 at a time through double-buffered LDS with the
// global loads of the following tiles in flight.  A batch of a thousand rows gives only 64 such
// tiles for 256 CUs, so the reduction dimension is also split across blocks; the fp32 partial
// tiles go to a workspace and a second small kernel adds them in a fixed order and applies bias
// and activation, which keeps the result reproducible.
#include "rec_common.h"

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef unsigned short ushort8 __attribute__((ext_vector_type(8)));

constexpr int GB_BM = 128, GB_BN = 128, GB_BK = 64;
constexpr int GB_THREADS = 256;
constexpr int GB_STAGES = 3;                              // k tiles of global loads in flight
constexpr int GB_LD = GB_BK + 8;                          // padded LDS row in bf16 elements (144 B)
constexpr int GB_TILE = (GB_BM + GB_BN) * GB_LD;          // elements per stage

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    const floatx2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));   // v_cvt_pk_bf16_f32, RNE
}

// Requires K % 64 == 0, lda % 4 == 0 (fp32 A) or % 8 == 0 (bf16 A), 16-byte aligned A and W.
// grid = ceil(N/128) * ceil(M/128) * S blocks.  S == 1: writes act(acc + bias) to C.  S > 1: k part z
// covers k in [z*K/S, (z+1)*K/S) and writes its raw fp32 tile to part[z][M][N].
template <bool A_BF16>
__global__ __launch_bounds__(GB_THREADS) void gemm_bf16_kernel(const void* __restrict__ Av, int64_t lda,
                                                               const uint16_t* __restrict__ W,
                                                               const float* __restrict__ bias, void* __restrict__ C,
                                                               int c_bf16, int64_t ldc, float* __restrict__ part, int M,
                                                               int N, int K, int S, int act) {
    __shared__ __attribute__((aligned(16))) uint16_t lds[2 * GB_TILE];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;
    // Blocks are dealt to the 8 XCDs round-robin.  Renumber them so that XCD x works on a
    // contiguous eighth of the (row tile, column tile, k part) list with the row tile slowest:
    // the x rows of one row tile are then fetched into a single L2 and reused by all its column
    // tiles there, instead of being fetched by eight L2s.
    int blk = blockIdx.x;
    {
        const int per = gridDim.x / 8;
        if (blk < per * 8) blk = (blk % 8) * per + blk / 8;
    }
    const int tiles_n = (N + GB_BN - 1) / GB_BN;
    const int z = blk % S;
    const int tile = blk / S;
    const int m0 = (tile / tiles_n) * GB_BM, n0 = (tile % tiles_n) * GB_BN;
    const int k_len = K / S;                              // host guarantees K % (S*64) == 0
    const int k_begin = z * k_len;
    const int n_tiles = k_len / GB_BK;

    // staging registers, GB_STAGES tiles deep: A tile 128x64 (fp32: 8 float4 per thread; bf16: 4 x 8
    // elements), W tile 4 x 8 elements
    struct StageRegs {
        float4 ra[A_BF16 ? 1 : 8];
        ushort8 rab[A_BF16 ? 4 : 1];
        ushort8 rw[4];
    };
    StageRegs st[GB_STAGES];

    auto load_tile = [&](StageRegs& r, int k0) __attribute__((always_inline)) {
        if constexpr (A_BF16) {
            const uint16_t* __restrict__ A = static_cast<const uint16_t*>(Av);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int f = tid + i * GB_THREADS, row = f >> 3, c = (f & 7) * 8;
                const int gr = m0 + row;
                r.rab[i] = *reinterpret_cast<const ushort8*>(A + (int64_t)(gr < M ? gr : 0) * lda + k0 + c);
            }
        } else {
            const float* __restrict__ A = static_cast<const float*>(Av);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int f = tid + i * GB_THREADS, row = f >> 4, c = (f & 15) * 4;
                const int gr = m0 + row;
                r.ra[i] = *reinterpret_cast<const float4*>(A + (int64_t)(gr < M ? gr : 0) * lda + k0 + c);
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int f = tid + i * GB_THREADS, row = f >> 3, c = (f & 7) * 8;
            const int gn = n0 + row;
            r.rw[i] = *reinterpret_cast<const ushort8*>(W + (int64_t)(gn < N ? gn : 0) * K + k0 + c);
        }
    };
    // rows past M / N were read from row 0 (a valid address); they only feed accumulator rows /
    // columns that are never stored, so no masking is needed
    auto store_tile = [&](const StageRegs& r, int s) __attribute__((always_inline)) {
        uint16_t* ta = lds + s * GB_TILE;
        uint16_t* tw = ta + GB_BM * GB_LD;
        if constexpr (A_BF16) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int f = tid + i * GB_THREADS, row = f >> 3, c = (f & 7) * 8;
                *reinterpret_cast<ushort8*>(ta + row * GB_LD + c) = r.rab[i];
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int f = tid + i * GB_THREADS, row = f >> 4, c = (f & 15) * 4;
                const uint2 o = make_uint2(pack_bf16(r.ra[i].x, r.ra[i].y), pack_bf16(r.ra[i].z, r.ra[i].w));
                *reinterpret_cast<uint2*>(ta + row * GB_LD + c) = o;
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int f = tid + i * GB_THREADS, row = f >> 3, c = (f & 7) * 8;
            *reinterpret_cast<ushort8*>(tw + row * GB_LD + c) = r.rw[i];
        }
    };

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = floatx16{0};

    const int frag = (lane & 31) * GB_LD + (lane >> 5) * 8;
    auto multiply_tile = [&](int cur) __attribute__((always_inline)) {
        const uint16_t* ta = lds + cur * GB_TILE + (wm * 64) * GB_LD + frag;
        const uint16_t* tw = lds + cur * GB_TILE + (GB_BM + wn * 64) * GB_LD + frag;
#pragma unroll
        for (int kc = 0; kc < GB_BK / 16; ++kc) {
            const bf16x8 a0 = *reinterpret_cast<const bf16x8*>(ta + kc * 16);
            const bf16x8 a1 = *reinterpret_cast<const bf16x8*>(ta + 32 * GB_LD + kc * 16);
            const bf16x8 b0 = *reinterpret_cast<const bf16x8*>(tw + kc * 16);
            const bf16x8 b1 = *reinterpret_cast<const bf16x8*>(tw + 32 * GB_LD + kc * 16);
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b1, acc[1][1], 0, 0, 0);
        }
    };
    // Every load in the steady-state loop is unconditional (a tile index past the end re-reads the
    // last tile and is never multiplied), so the number of loads in flight at each point is fixed
    // and the hardware wait counters can let the younger GB_STAGES-1 tiles stay outstanding while
    // the oldest is written to LDS.  Conditional loads would force a wait for all of them.
    const int last_tile = n_tiles - 1;
    auto tile_k = [&](int t) { return k_begin + (t < last_tile ? t : last_tile) * GB_BK; };
#pragma unroll
    for (int p = 0; p < GB_STAGES; ++p) load_tile(st[p], tile_k(p));
    store_tile(st[0], 0);
    __syncthreads();
    const int full_groups = n_tiles / GB_STAGES;
    for (int g = 0; g < full_groups; ++g) {
#pragma unroll
        for (int p = 0; p < GB_STAGES; ++p) {
            const int it = g * GB_STAGES + p;
            const int cur = it & 1;
            load_tile(st[p], tile_k(it + GB_STAGES));           // stage p went to LDS one step ago
            multiply_tile(cur);
            // keep the conversion of the next tile (which waits for its loads) behind the multiply:
            // hoisted above it, the wait would stall the matrix cores on memory latency
            __builtin_amdgcn_sched_barrier(0);
            store_tile(st[(p + 1) % GB_STAGES], cur ^ 1);       // tile it+1
            __syncthreads();
        }
    }
    // the n_tiles % GB_STAGES tiles left over are already in st[0..] / LDS; no loads here
#pragma unroll
    for (int p = 0; p < GB_STAGES - 1; ++p) {
        const int it = full_groups * GB_STAGES + p;
        if (it < n_tiles) {
            const int cur = it & 1;
            multiply_tile(cur);
            if (it + 1 < n_tiles) store_tile(st[p + 1], cur ^ 1);
            __syncthreads();
        }
    }

    // MFMA 32x32 accumulator layout: register v of lane l holds row 8*(v/4) + 4*(l/32) + v%4, col l%32
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = n0 + wn * 64 + j * 32 + (lane & 31);
            if (n >= N) continue;
            const float bv = (S == 1) ? bias[n] : 0.f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm * 64 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (m >= M) continue;
                if (S == 1) {
                    const float z = rec_apply_act(acc[i][j][v] + bv, act);
                    if (c_bf16) static_cast<uint16_t*>(C)[(int64_t)m * ldc + n] = rec_f32_to_bf16_bits(z);
                    else static_cast<float*>(C)[(int64_t)m * ldc + n] = z;
                } else {
                    part[((int64_t)z * M + m) * N + n] = acc[i][j][v];
                }
            }
        }
    }
}

// C = act(sum_z part[z] + bias), z = 0, 1, ... in order.  One thread per 4 consecutive columns.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ part, int S,
                                                            const float* __restrict__ bias, void* __restrict__ C,
                                                            int c_bf16, int64_t ldc, int M, int N, int act) {
    const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;      // quad index
    const int nq = (N + 3) / 4;
    if (q >= (int64_t)M * nq) return;
    const int m = (int)(q / nq), n = (int)(q - (int64_t)m * nq) * 4;
    float s[4] = {0.f, 0.f, 0.f, 0.f};
    const bool full = (n + 3 < N) && (N % 4 == 0);
    for (int z = 0; z < S; ++z) {
        const float* p = part + ((int64_t)z * M + m) * N + n;
        if (full) {
            const float4 v = *reinterpret_cast<const float4*>(p);
            s[0] += v.x; s[1] += v.y; s[2] += v.z; s[3] += v.w;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (n + e < N) s[e] += p[e];
        }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (n + e < N) {
            const float z = rec_apply_act(s[e] + bias[n + e], act);
            if (c_bf16) static_cast<uint16_t*>(C)[(int64_t)m * ldc + n + e] = rec_f32_to_bf16_bits(z);
            else static_cast<float*>(C)[(int64_t)m * ldc + n + e] = z;
        }
    }
}

}  // namespace

// Split factor for the cross-block k split: enough blocks for the 256 CUs, k parts of at least
// 256 that are multiples of the 64-wide step.  Returns 0 if the large-tile kernel does not apply.
int rec_gemm_bf16_split(int M, int N, int K) {
    if (K % GB_BK != 0 || K < 256) return 0;
    const int64_t tiles = (int64_t)((M + GB_BM - 1) / GB_BM) * ((N + GB_BN - 1) / GB_BN);
    if (tiles < 64) return 0;                 // smaller layers do better on the 64x64 / 32x32 kernels
    int S = 1;
    while (S < 8 && tiles * S < 256 && K % (S * 2 * GB_BK) == 0 && K / (S * 2) >= 256) S *= 2;
    return S;
}

size_t rec_gemm_bf16_partial_bytes(int M, int N, int K) {
    const int S = rec_gemm_bf16_split(M, N, K);
    return S > 1 ? rec_round_up((size_t)S * M * N * sizeof(float), 256) : 0;
}

rec_status rec_gemm_bf16_launch(const void* x, bool x_bf16, int64_t ldx, const void* W, const float* bias, void* y,
                                bool y_bf16, int64_t ldy, float* partial, int M, int N, int K, int act,
                                hipStream_t s) {
    const int S = rec_gemm_bf16_split(M, N, K);
    if (S < 1) return REC_ERR_UNSUPPORTED;
    if (S > 1 && !partial) return REC_ERR_WORKSPACE;
    const dim3 grid((unsigned)(((N + GB_BN - 1) / GB_BN) * ((M + GB_BM - 1) / GB_BM) * S)), block(GB_THREADS);
    const uint16_t* Wb = static_cast<const uint16_t*>(W);
    if (x_bf16)
        hipLaunchKernelGGL(gemm_bf16_kernel<true>, grid, block, 0, s, x, ldx, Wb, bias, y, (int)y_bf16, ldy, partial, M, N,
                           K, S, act);
    else
        hipLaunchKernelGGL(gemm_bf16_kernel<false>, grid, block, 0, s, x, ldx, Wb, bias, y, (int)y_bf16, ldy, partial, M, N,
                           K, S, act);
    REC_CHECK_LAUNCH();
    if (S > 1) {
        const int64_t quads = (int64_t)M * ((N + 3) / 4);
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, s, partial, S, bias,
                           y, (int)y_bf16, ldy, M, N, act);
        REC_CHECK_LAUNCH();
    }
    return REC_OK;
}
