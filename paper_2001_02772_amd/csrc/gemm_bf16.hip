// Large FC layers on the matrix cores: C = act(A W^T + b) with A [M x K], W [N x K], fp32 accumulate; bf16 operands
// on every tile shape, fp32 operands on the small-tile kernel.
//
// This is the one genuinely dense, FLOP-heavy contraction of the models in Table I of the
// DeepRecSys paper: the first Dense-FC layer of the MLP-dominated DLRM-RMC3 (thousands of dense
// inputs into a 1024-wide layer; Section III-A: its run time is dominated by FC layers).
//
// Both operands are contiguous along k, so a 64-wide k slice of a row is one 128-byte line.  Tiles
// go from global memory straight into LDS (global_load_lds_dwordx4: no staging registers, so the
// register file holds accumulators and operand fragments only); a wave instruction moves 8 rows x
// 128 bytes, and the 16-byte chunks of a row are XOR-swizzled with half the row number -- applied on the
// global side, because the LDS side of such a load is lane-linear -- so that the 16-byte fragment
// reads of the 32x32x16 MFMA are bank-conflict free without padding.  A ring of NST stages keeps
// several k slices in flight; the wave waits with explicit vmcnt counts, and the one barrier per
// slice sits in the middle of the slice (NST >= 3) so the next slice's first fragments are read
// while the current slice still multiplies.  Measured on the part: LDS delivers 128 bytes/clock per
// CU, so a wave must own at least a 64x64 sub-tile (2x2 MFMA tiles) for the matrix cores not to wait
// on fragment reads, and a CU fetches about 70-100 GB/s from L2, which is why the large-batch
// variant uses 256x256 tiles.
//
// The tile shrinks with the batch so that there is about a block per CU: 256x256 (8 waves), 128x128,
// 128x64 or 64x64 (4 waves).  At a batch of a thousand rows the 64x64 tiles re-fetch each operand
// sixteen times from L2 and the layer is bound by what a CU can fetch, not by the matrix cores;
// splitting k across blocks instead (128x128 tiles, partial tiles through memory, the last arrival
// folding them) was measured no faster, because making the partial tiles visible across the XCDs'
// separate L2s needs device-scope fences that cost more than the fetches they save.
#include "rec_common.h"
#include "scan_body.h"

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// 64 lanes x 16 bytes from global (uniform base + per-lane byte offset) to LDS: lane l's bytes land at
// LDS address lds_off + 16 l.  Tracked by vmcnt like any vector load.
__device__ __forceinline__ void lds_dma16(uint32_t lane_off, const void* base, uint32_t lds_off) {
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1\n" ::"v"(lane_off), "s"(base), "s"(lds_off) : "memory");
}
// Wait until at most N of this wave's vector loads are outstanding, then meet the block's other
// waves.  One asm statement with a memory clobber: no LDS access moves across it.
template <int N>
__device__ __forceinline__ void wait_loads_barrier() {
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}
// The same with a count known only at run time (block-uniform): at most min(r, MAXR) groups of LPT loads.
template <int LPT, int MAXR>
__device__ __forceinline__ void wait_groups_barrier(int r) {
    if constexpr (MAXR == 0) {
        wait_loads_barrier<0>();
    } else {
        if (r >= MAXR) wait_loads_barrier<MAXR * LPT>();
        else wait_groups_barrier<LPT, MAXR - 1>(r);
    }
}
template <int N>
__device__ __forceinline__ void wait_loads_lds_barrier() {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

// Slot of a 16-byte chunk inside its 128-byte LDS row: chunk ^ swz(row).  LDS has 64 banks of 4 bytes
// and serves a 16-byte read 16 lanes at a time; the lanes of an MFMA fragment read take the same
// chunk of 16 consecutive rows, which this spreads over all 16 bank groups (rows alternate between the
// two 128-byte halves of the bank range, row pairs take the 8 slots).  Checked with the LDS bank
// conflict counter: 4 cycles per read instruction, against 8 with chunk ^ (row % 8).
__device__ __forceinline__ int swz(int row) { return (row >> 1) & 7; }

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    const floatx2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));   // v_cvt_pk_bf16_f32, RNE
}

template <int BM_, int BN_, int WM_, int WN_, int NST_>
struct GemmCfg {
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, NST = NST_;
    static constexpr int NW = WM * WN, THREADS = 64 * NW;
    static constexpr int TM = BM / WM / 32, TN = BN / WN / 32;          // MFMA tiles per wave
    static constexpr int STAGE_BYTES = (BM + BN) * 128;                 // one 64-wide k slice of both operands
    static constexpr int A_PER_WAVE = BM / 8 / NW, W_PER_WAVE = BN / 8 / NW;
    static constexpr int LPT = A_PER_WAVE + W_PER_WAVE;                 // load instructions per wave per slice
    static constexpr int ACC = TM * TN * 16;                            // accumulator floats per thread
    static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "tile rows must split evenly over the waves");
    static_assert(NST * STAGE_BYTES <= 160 * 1024, "LDS capacity");
    static_assert((NST - 1) * LPT < 64, "vmcnt is a 6-bit counter");
};

// act(acc + bias) for a wave's TM x TN MFMA tiles whose top-left element is (row0, col0).
// MFMA 32x32 accumulator layout: register v of lane l holds row 8 (v/4) + 4 (l/32) + v%4, column l%32.
// Bias values are fetched before the first store so that no load waits behind the stores.
template <bool C_BF16, int TM, int TN>
__device__ __forceinline__ void store_tiles(const floatx16 (&acc)[TM][TN], const float* __restrict__ bias,
                                            void* __restrict__ Cv, int64_t ldc, int M, int N, int row0, int col0, bool full,
                                            int lane, int act) {
    typedef typename std::conditional<C_BF16, uint16_t, float>::type out_t;
    out_t* Cp = static_cast<out_t*>(Cv);
    float bv[TN];
    int nn[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        nn[j] = col0 + j * 32 + (lane & 31);
        bv[j] = nn[j] < N ? bias[nn[j]] : 0.f;
    }
    const bool relu = act == REC_ACT_RELU, sigm = act == REC_ACT_SIGMOID;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int mb = row0 + i * 32 + 4 * (lane >> 5);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            out_t* col = Cp + nn[j];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = mb + 8 * (v >> 2) + (v & 3);
                float zv = acc[i][j][v] + bv[j];
                if (relu) zv = fmaxf(zv, 0.f);
                if (sigm) zv = 1.0f / (1.0f + expf(-zv));
                if (full || (m < M && nn[j] < N)) {
                    if constexpr (C_BF16) col[(int64_t)m * ldc] = (uint16_t)pack_bf16(zv, 0.f);
                    else col[(int64_t)m * ldc] = zv;
                }
            }
        }
    }
}

// Requires K % 64 == 0, 16-byte aligned A and W, lda and ldw multiples of 8, M*lda*2 and N*ldw*2
// below 2^32.  grid = tiles_m * tiles_n blocks.
template <class C, bool C_BF16>
__global__ __launch_bounds__(C::THREADS) void gemm_bf16_kernel(const uint16_t* __restrict__ A, int64_t lda,
                                                               const uint16_t* __restrict__ W, int64_t ldw,
                                                               const float* __restrict__ bias, void* __restrict__ Cv,
                                                               int64_t ldc, int M, int N, int K, int act) {
    constexpr int BM = C::BM, BN = C::BN, NST = C::NST, TM = C::TM, TN = C::TN;
    __shared__ __attribute__((aligned(1024))) unsigned char lds[NST * C::STAGE_BYTES];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % C::WM, wn = wave / C::WM;

    // Blocks are dealt to the 8 XCDs round-robin.  Renumber them so that XCD x works on a contiguous
    // eighth of the (row tile, column tile) list, row tile slowest: a few whole row tiles per XCD, whose
    // operand slices then live in that XCD's L2 and are shared by its CUs.
    int o = blockIdx.x;
    {
        const int per = gridDim.x / 8;
        if (o < per * 8) o = (o % 8) * per + o / 8;
    }
    const int tiles_n = (N + BN - 1) / BN, tiles_m = (M + BM - 1) / BM, tiles = tiles_m * tiles_n;
    const int tile = o < tiles ? o : tiles - 1;
    const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;
    const int n_slices = K / 64;

    // Load instruction j of a wave covers tile rows (j NW + wave) 8 .. +8; lane l fetches, for row
    // r = that + l/8, the chunk (l%8) ^ swz(r) and deposits it in slot l%8 of the row.  Rows past the
    // matrix edge re-read the last row (a valid address); they only feed results that are not stored.
    uint32_t offA[C::A_PER_WAVE], offW[C::W_PER_WAVE];
#pragma unroll
    for (int j = 0; j < C::A_PER_WAVE; ++j) {
        const int r = (j * C::NW + wave) * 8 + (lane >> 3);
        const int gr = min(m0 + r, M - 1);
        offA[j] = (uint32_t)((int64_t)gr * lda * 2 + (((lane & 7) ^ swz(r)) * 16));
    }
#pragma unroll
    for (int j = 0; j < C::W_PER_WAVE; ++j) {
        const int r = (j * C::NW + wave) * 8 + (lane >> 3);
        const int gr = min(n0 + r, N - 1);
        offW[j] = (uint32_t)((int64_t)gr * ldw * 2 + (((lane & 7) ^ swz(r)) * 16));
    }
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds;
    const unsigned char* gA = reinterpret_cast<const unsigned char*>(A);
    const unsigned char* gW = reinterpret_cast<const unsigned char*>(W);
    auto request = [&](int slice, int stage) __attribute__((always_inline)) {
        const unsigned char* a = gA + (int64_t)slice * 128;
        const unsigned char* w = gW + (int64_t)slice * 128;
        const uint32_t sb = lds_base + stage * C::STAGE_BYTES + wave * 1024;
#pragma unroll
        for (int j = 0; j < C::A_PER_WAVE; ++j) lds_dma16(offA[j], a, sb + j * C::NW * 1024);
#pragma unroll
        for (int j = 0; j < C::W_PER_WAVE; ++j) lds_dma16(offW[j], w, sb + BM * 128 + j * C::NW * 1024);
    };

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = floatx16{0};

    // MFMA 32x32x16 operands: lane l supplies row l%32 and the 8 k values of chunk 2 kc + l/32.
    const int ra = wm * (BM / C::WM) + (lane & 31), rw = wn * (BN / C::WN) + (lane & 31);
    const int fa = swz(ra), fw = swz(rw), hi = lane >> 5;
    bf16x8 af[2][TM], wf[2][TN];
    auto load_frags = [&](int stage, int kc, int buf) __attribute__((always_inline)) {
        const unsigned char* sa = lds + stage * C::STAGE_BYTES + ra * 128;
        const unsigned char* sw = lds + stage * C::STAGE_BYTES + BM * 128 + rw * 128;
#pragma unroll
        for (int i = 0; i < TM; ++i) af[buf][i] = *reinterpret_cast<const bf16x8*>(sa + i * 4096 + (((2 * kc + hi) ^ fa) * 16));
#pragma unroll
        for (int j = 0; j < TN; ++j) wf[buf][j] = *reinterpret_cast<const bf16x8*>(sw + j * 4096 + (((2 * kc + hi) ^ fw) * 16));
    };
    auto multiply = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[buf][i], wf[buf][j], acc[i][j], 0, 0, 0);
    };

    if constexpr (NST >= 3) {
        // Slice t lives in stage t % NST.  In the middle of slice t: slice t+1 has landed (own loads
        // waited for, then the barrier), and every wave is past slice t-1, so its stage takes the request
        // for slice t+NST-1.  The wait counts are the wave's own requests issued after the awaited one.
#pragma unroll
        for (int p = 0; p < NST - 1; ++p)
            if (p < n_slices) request(p, p);
        wait_groups_barrier<C::LPT, NST - 2>(n_slices - 1);          // slice 0 landed; up to NST-2 younger ones in flight
        load_frags(0, 0, 0);
        for (int t0 = 0; t0 < n_slices; t0 += NST) {
#pragma unroll
            for (int s = 0; s < NST; ++s) {
                const int t = t0 + s;
                if (t < n_slices) {
                    load_frags(s, 1, 1);
                    multiply(0);
                    load_frags(s, 2, 0);
                    multiply(1);
                    if (t + 1 < n_slices) {
                        // in flight: slices t+1 .. min(t+NST-2, n_slices-1); t+1 must be complete
                        wait_groups_barrier<C::LPT, NST - 3>(n_slices - 2 - t);
                        if (t + NST - 1 < n_slices) request(t + NST - 1, (s + NST - 1) % NST);
                    }
                    load_frags(s, 3, 1);
                    multiply(0);
                    if (t + 1 < n_slices) load_frags((s + 1) % NST, 0, 0);
                    multiply(1);
                }
            }
        }
    } else {
        // two stages: slice t+1 is requested as soon as every wave has left slice t-1
        request(0, 0);
        for (int t0 = 0; t0 < n_slices; t0 += 2) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const int t = t0 + s;
                if (t < n_slices) {
                    wait_loads_lds_barrier<0>();
                    if (t + 1 < n_slices) request(t + 1, s ^ 1);
                    load_frags(s, 0, 0);
                    load_frags(s, 1, 1);
                    multiply(0);
                    load_frags(s, 2, 0);
                    multiply(1);
                    load_frags(s, 3, 1);
                    multiply(0);
                    multiply(1);
                }
            }
        }
    }

    store_tiles<C_BF16, TM, TN>(acc, bias, Cv, ldc, M, N, m0 + wm * (BM / C::WM), n0 + wn * (BN / C::WN),
                                (m0 + BM <= M) && (n0 + BN <= N), lane, act);
}

// Small tiles (64x64 or 64x32) with the four waves splitting k instead of the tile: wave w multiplies
// the whole tile for the w-th quarter of every 128-byte k slice, so a slice of a 64x64 tile costs 16 KiB
// of fragment reads instead of 32 (with the 16 KiB the loads write, LDS traffic per slice drops by a
// third, and at this tile size LDS is what the bf16 matrix cores wait for).  The four partial tiles meet
// in LDS at the end and are added in wave order, one 32x32 MFMA tile per wave.
// F32: operands are fp32 (a slice is 32 k wide) and go through v_mfma_f32_32x32x2_f32: a lane's 16-byte
// fragment holds 4 consecutive k, component e of the two lane halves feeds MFMA e -- activations and
// weights use the same assignment, so every k is multiplied exactly once.  The fp32 matrix rate is a
// sixteenth of the bf16 one, which makes such a layer compute-bound and the tile as small as it takes
// to give every CU a block.  Requirements as for gemm_bf16_kernel, with K % 32 == 0 for fp32.
template <int TM, int TN, int NST, bool F32, bool C_BF16>
__global__ __launch_bounds__(256) void gemm_ks_kernel(const void* __restrict__ A, int64_t lda, const void* __restrict__ W,
                                                     int64_t ldw, const float* __restrict__ bias, void* __restrict__ Cv,
                                                     int64_t ldc, int M, int N, int K, int act) {
    constexpr int BM = 32 * TM, BN = 32 * TN, STAGE_BYTES = (BM + BN) * 128, LPT = TM + TN;
    constexpr int ELT = F32 ? 4 : 2, KS = 128 / ELT;           // bytes per element, k per slice
    static_assert(NST % 2 == 0 && NST >= 4 && NST * STAGE_BYTES >= 4 * TM * TN * 16 * 64 * 4, "ring doubles as the fold buffer");
    static_assert(NST * STAGE_BYTES <= 160 * 1024 && (NST - 1) * LPT < 64 && TM * TN <= 4, "LDS, vmcnt, one tile per wave in the fold");
    __shared__ __attribute__((aligned(1024))) unsigned char lds[NST * STAGE_BYTES];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    int o = blockIdx.x;
    {
        const int per = gridDim.x / 8;
        if (o < per * 8) o = (o % 8) * per + o / 8;
    }
    const int tiles_n = (N + BN - 1) / BN;
    const int m0 = (o / tiles_n) * BM, n0 = (o % tiles_n) * BN;
    const int n_slices = K / KS;

    uint32_t offA[TM], offW[TN];
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        const int r = (j * 4 + wave) * 8 + (lane >> 3);
        offA[j] = (uint32_t)((int64_t)min(m0 + r, M - 1) * lda * ELT + (((lane & 7) ^ swz(r)) * 16));
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int r = (j * 4 + wave) * 8 + (lane >> 3);
        offW[j] = (uint32_t)((int64_t)min(n0 + r, N - 1) * ldw * ELT + (((lane & 7) ^ swz(r)) * 16));
    }
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds;
    const unsigned char* gA = static_cast<const unsigned char*>(A);
    const unsigned char* gW = static_cast<const unsigned char*>(W);
    auto request = [&](int slice, int stage) __attribute__((always_inline)) {
        const uint32_t sb = lds_base + stage * STAGE_BYTES + wave * 1024;
#pragma unroll
        for (int j = 0; j < TM; ++j) lds_dma16(offA[j], gA + (int64_t)slice * 128, sb + j * 4096);
#pragma unroll
        for (int j = 0; j < TN; ++j) lds_dma16(offW[j], gW + (int64_t)slice * 128, sb + BM * 128 + j * 4096);
    };

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = floatx16{0};
    const int row = lane & 31, hi = lane >> 5;
    const int chunk = ((2 * wave + hi) ^ swz(row)) * 16;       // this wave's quarter of every slice
    float4 af[2][TM], wf[2][TN];                                // 16-byte fragments (8 bf16 or 4 fp32)
    auto load_frags = [&](int stage, int buf) __attribute__((always_inline)) {
        const unsigned char* sa = lds + stage * STAGE_BYTES + row * 128 + chunk;
#pragma unroll
        for (int i = 0; i < TM; ++i) af[buf][i] = *reinterpret_cast<const float4*>(sa + i * 4096);
#pragma unroll
        for (int j = 0; j < TN; ++j) wf[buf][j] = *reinterpret_cast<const float4*>(sa + BM * 128 + j * 4096);
    };
    auto multiply = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if constexpr (F32) {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[buf][i].x, wf[buf][j].x, acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[buf][i].y, wf[buf][j].y, acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[buf][i].z, wf[buf][j].z, acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[buf][i].w, wf[buf][j].w, acc[i][j], 0, 0, 0);
                } else {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, af[buf][i]),
                                                                        __builtin_bit_cast(bf16x8, wf[buf][j]), acc[i][j], 0, 0, 0);
                }
            }
    };

#pragma unroll
    for (int p = 0; p < NST - 1; ++p)
        if (p < n_slices) request(p, p);
    wait_groups_barrier<LPT, NST - 2>(n_slices - 1);
    load_frags(0, 0);
    for (int t0 = 0; t0 < n_slices; t0 += NST) {
#pragma unroll
        for (int s = 0; s < NST; ++s) {
            const int t = t0 + s;
            if (t < n_slices) {
                if (t + 1 < n_slices) {
                    // slice t+1 has landed; every wave is past slice t-1, whose stage takes slice t+NST-1
                    wait_groups_barrier<LPT, NST - 3>(n_slices - 2 - t);
                    if (t + NST - 1 < n_slices) request(t + NST - 1, (s + NST - 1) % NST);
                    load_frags((s + 1) % NST, (s + 1) & 1);
                }
                multiply(s & 1);
            }
        }
    }

    // fold: partial tiles to LDS as [wave][register][lane], then wave q sums MFMA tile q in wave order
    wait_loads_lds_barrier<0>();                               // nobody still reads the ring
    float* red = reinterpret_cast<float*>(lds);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) red[((wave * (TM * TN) + i * TN + j) * 16 + v) * 64 + lane] = acc[i][j][v];
    __syncthreads();
    if (wave >= TM * TN) return;
    floatx16 sum[1][1];
    sum[0][0] = floatx16{0};
#pragma unroll
    for (int w = 0; w < 4; ++w)
#pragma unroll
        for (int v = 0; v < 16; ++v) sum[0][0][v] += red[((w * (TM * TN) + wave) * 16 + v) * 64 + lane];
    const int qi = wave / TN, qj = wave % TN;
    store_tiles<C_BF16, 1, 1>(sum, bias, Cv, ldc, M, N, m0 + qi * 32, n0 + qj * 32, (m0 + BM <= M) && (n0 + BN <= N), lane, act);
}

// fp32 rows -> bf16 rows (round to nearest even), 8 elements per thread; the first `scan_tiles`
// blocks do a bag-offsets scan instead.
__global__ __launch_bounds__(SCAN_THREADS) void prepare_bf16_kernel(const float* __restrict__ x, int64_t ldx,
                                                                    uint16_t* __restrict__ y, int64_t ldy, int32_t M,
                                                                    int32_t K, const int32_t* __restrict__ len,
                                                                    int64_t n_bags, int64_t* __restrict__ off, int vec_ok,
                                                                    int scan_tiles) {
    if ((int)blockIdx.x < scan_tiles) {
        offsets_block(len, n_bags, off, vec_ok, (int)blockIdx.x, true);
        return;
    }
    const int k8 = K / 8;
    const int64_t n8 = (int64_t)M * k8;
    const int64_t step = (int64_t)(gridDim.x - scan_tiles) * SCAN_THREADS;
    constexpr int U = 2;                                       // items per thread per round, loads first
    for (int64_t i0 = (int64_t)(blockIdx.x - scan_tiles) * SCAN_THREADS + threadIdx.x; i0 < n8; i0 += U * step) {
        float4 a[U], b[U];
        int64_t dst[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = i0 + u * step;
            const int64_t m = (i < n8 ? i : i0) / k8;
            const int c = (int)((i < n8 ? i : i0) - m * k8) * 8;
            a[u] = *reinterpret_cast<const float4*>(x + m * ldx + c);
            b[u] = *reinterpret_cast<const float4*>(x + m * ldx + c + 4);
            dst[u] = i < n8 ? m * ldy + c : -1;
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (dst[u] >= 0)
                *reinterpret_cast<uint4*>(y + dst[u]) = make_uint4(pack_bf16(a[u].x, a[u].y), pack_bf16(a[u].z, a[u].w),
                                                                   pack_bf16(b[u].x, b[u].y), pack_bf16(b[u].z, b[u].w));
    }
}

// Tile shapes, largest first; a shape is taken when it gives about a block per CU.  Below these comes
// the 64x64 tile of gemm_ks_kernel (8 stages of 16 KiB).
typedef GemmCfg<256, 256, 4, 2, 2> Cfg256;      // 8 waves of 64x128, 2 stages of 64 KiB
typedef GemmCfg<128, 128, 2, 2, 4> Cfg128;      // 4 waves of 64x64, 4 stages of 32 KiB
typedef GemmCfg<128, 64, 2, 2, 5> Cfg128x64;    // 4 waves of 64x32, 5 stages of 24 KiB

constexpr int GEMM_MIN_BLOCKS = 200;      // about one block per CU

int64_t tile_count(int M, int N, int bm, int bn) { return (int64_t)((M + bm - 1) / bm) * ((N + bn - 1) / bn); }

}  // namespace

rec_gemm_plan rec_gemm_bf16_plan(int M, int N, int K) {
    rec_gemm_plan p = {0, 0, 0};
    if (M < 1 || N < 1 || K < 256 || K % 64 != 0) return p;
    if ((int64_t)M * K * 2 >= (int64_t)1 << 32 || (int64_t)N * K * 2 >= (int64_t)1 << 32) return p;
    const int shapes[4][2] = {{256, 256}, {128, 128}, {128, 64}, {64, 64}};
    for (int i = 0; i < 4; ++i) {
        const int64_t t = tile_count(M, N, shapes[i][0], shapes[i][1]);
        // the smallest shape also serves layers that leave part of the device idle, down to a quarter
        if (t >= GEMM_MIN_BLOCKS || (i == 3 && t >= 64)) {
            p.bm = shapes[i][0];
            p.bn = shapes[i][1];
            p.tiles = (int)t;
            return p;
        }
    }
    return p;
}

// Workspace of one layer launch: the bf16 copy of fp32 activations (none for bf16 input).
size_t rec_gemm_bf16_workspace_bytes(int M, int N, int K, bool x_bf16) {
    (void)N;
    return x_bf16 ? 0 : rec_round_up((size_t)M * K * sizeof(uint16_t), 256);
}

rec_status rec_gemm_bf16_launch(const void* x, bool x_bf16, int64_t ldx, const void* W, const float* bias, void* y,
                                bool y_bf16, int64_t ldy, void* workspace, int M, int N, int K, int act,
                                const rec_scan_job* scan, hipStream_t s) {
    const rec_gemm_plan p = rec_gemm_bf16_plan(M, N, K);
    if (p.tiles == 0) return REC_ERR_UNSUPPORTED;
    if (!workspace && !x_bf16) return REC_ERR_WORKSPACE;
    uint16_t* xh = static_cast<uint16_t*>(workspace);

    int scan_tiles = 0;
    if (scan) {
        scan_tiles = rec_scan_parallel_tiles(scan->n);
        if (scan_tiles < 1) return REC_ERR_BAD_SHAPE;          // the caller launches such a scan itself
    }
    if (!x_bf16 || scan_tiles > 0) {
        // one preparing launch: bf16 copy of the activations, and the scan if one rides along
        const int64_t n8 = x_bf16 ? 0 : (int64_t)M * (K / 8);
        int64_t blocks = (n8 + 2 * SCAN_THREADS - 1) / (2 * SCAN_THREADS);        // two items per thread
        blocks = blocks < 1 ? 1 : (blocks > 4096 ? 4096 : blocks);
        hipLaunchKernelGGL(prepare_bf16_kernel, dim3((unsigned)(blocks + scan_tiles)), dim3(SCAN_THREADS), 0, s,
                           static_cast<const float*>(x), ldx, xh, (int64_t)K, x_bf16 ? 0 : M, K,
                           scan ? scan->lengths : nullptr, scan ? scan->n : 0, scan ? scan->offsets : nullptr,
                           scan ? (int)rec_aligned(scan->lengths, 16) : 0, scan_tiles);
        REC_CHECK_LAUNCH();
    }
    const uint16_t* Ab = x_bf16 ? static_cast<const uint16_t*>(x) : xh;
    const int64_t lda = x_bf16 ? ldx : (int64_t)K;
    const uint16_t* Wb = static_cast<const uint16_t*>(W);
#define GEMM_GO(CFG)                                                                                                    \
    do {                                                                                                                \
        const dim3 grid((unsigned)p.tiles), block(CFG::THREADS);                                                        \
        if (y_bf16)                                                                                                     \
            hipLaunchKernelGGL((gemm_bf16_kernel<CFG, true>), grid, block, 0, s, Ab, lda, Wb, (int64_t)K, bias, y, ldy, M, N, K, act); \
        else                                                                                                            \
            hipLaunchKernelGGL((gemm_bf16_kernel<CFG, false>), grid, block, 0, s, Ab, lda, Wb, (int64_t)K, bias, y, ldy, M, N, K, act); \
    } while (0)
    if (p.bm == 256) GEMM_GO(Cfg256);
    else if (p.bm == 128 && p.bn == 128) GEMM_GO(Cfg128);
    else if (p.bm == 128) GEMM_GO(Cfg128x64);
    else if (y_bf16)
        hipLaunchKernelGGL((gemm_ks_kernel<2, 2, 8, false, true>), dim3((unsigned)p.tiles), dim3(256), 0, s, Ab, lda, Wb, (int64_t)K,
                           bias, y, ldy, M, N, K, act);
    else
        hipLaunchKernelGGL((gemm_ks_kernel<2, 2, 8, false, false>), dim3((unsigned)p.tiles), dim3(256), 0, s, Ab, lda, Wb, (int64_t)K,
                           bias, y, ldy, M, N, K, act);
#undef GEMM_GO
    REC_CHECK_LAUNCH();
    return REC_OK;
}

// ---- fp32 layers on the same machinery -------------------------------------------------------------
rec_gemm_plan rec_gemm_f32_plan(int M, int N, int K) {
    rec_gemm_plan p = {0, 0, 0};
    if (M < 1 || N < 1 || K < 256 || K % 32 != 0) return p;
    if ((int64_t)M * K * 4 >= (int64_t)1 << 32 || (int64_t)N * K * 4 >= (int64_t)1 << 32) return p;
    const int64_t t64 = tile_count(M, N, 64, 64), t6432 = tile_count(M, N, 64, 32);
    if (t64 >= GEMM_MIN_BLOCKS) {
        p.bm = 64, p.bn = 64, p.tiles = (int)t64;
    } else if (t6432 >= 128) {
        p.bm = 64, p.bn = 32, p.tiles = (int)t6432;
    }
    return p;
}

rec_status rec_gemm_f32_launch(const float* x, int64_t ldx, const float* W, const float* bias, float* y, int64_t ldy, int M,
                               int N, int K, int act, hipStream_t s) {
    const rec_gemm_plan p = rec_gemm_f32_plan(M, N, K);
    if (p.tiles == 0) return REC_ERR_UNSUPPORTED;
    if (p.bn == 64)
        hipLaunchKernelGGL((gemm_ks_kernel<2, 2, 8, true, false>), dim3((unsigned)p.tiles), dim3(256), 0, s, x, ldx, W, (int64_t)K, bias,
                           y, ldy, M, N, K, act);
    else
        hipLaunchKernelGGL((gemm_ks_kernel<2, 1, 8, true, false>), dim3((unsigned)p.tiles), dim3(256), 0, s, x, ldx, W, (int64_t)K, bias,
                           y, ldy, M, N, K, act);
    REC_CHECK_LAUNCH();
    return REC_OK;
}
