// Embedding lookup + sum pooling for all tables in one launch, the offsets scan
// that feeds it, and the sparse-input validator.
//
// Section II-A ("Embedding Table Access") of the DeepRecSys paper: every sparse
// feature indexes rows of its embedding table and the rows are combined by a
// pooling operation; Table I fixes the pooling of the DLRM-RMC models to Sum
// with about 80 (RMC1/2) or 20 (RMC3) lookups per table.  Sections III-A and
// VI-A name this the memory-bound, irregular part, so the kernel is organised
// around keeping many independent 16-byte row loads in flight per wavefront.
#include <mutex>

#include "rec_common.h"
#include "scan_body.h"

namespace {

// ------------------------------------------------------------------ offsets scan
__global__ __launch_bounds__(SCAN_THREADS) void offsets_kernel(const int32_t* __restrict__ len, int64_t n,
                                                               int64_t* __restrict__ off, int vec_ok) {
    offsets_block(len, n, off, vec_ok, (int)blockIdx.x, gridDim.x > 1);
}

// ------------------------------------------------------------------ SLS
// One wavefront per bag.  A row of D floats is covered by LPR lanes holding a
// float4 each, so one load instruction fetches RPI = 64/LPR rows; U such loads
// are issued back to back before any add, so a wave keeps U*RPI rows in flight.
// The bag's indices are read once, coalesced, 64 at a time, and handed to the
// row groups with a cross-lane read.  The RPI partial sums are folded with xor
// shuffles at the end; the add order is fixed, so results are reproducible.
constexpr int SLS_WAVES_PER_BLOCK = 4;

template <int LPR, int U>
__global__ __launch_bounds__(SLS_WAVES_PER_BLOCK* REC_WAVE) void sls_kernel(
    const float* const* __restrict__ tables, const int32_t* __restrict__ indices,
    const int64_t* __restrict__ off, int64_t n_bags, int32_t B, int32_t D, float* __restrict__ out,
    int64_t stride_b, int64_t stride_t) {
    constexpr int RPI = REC_WAVE / LPR;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    // Workgroups are handed to the 8 XCDs round-robin.  Renumbered, XCD x walks a contiguous
    // eighth of the bag range (= a few whole tables, bags being table-major), so the rows that
    // are popular in a table are fetched into one L2 instead of eight.  Measured with L2 request
    // counters on the embedding-dominated model with Zipf(1.05) indices: reads from memory drop
    // from 375 MB to 267 MB per batch (the rows a batch touches are 244 MB), L2 hit rate 41 -> 54 %.
    int64_t blk = blockIdx.x;
    {
        const int64_t per = gridDim.x / 8;
        if (blk < per * 8) blk = (blk % 8) * per + blk / 8;
    }
    const int64_t bag = blk * SLS_WAVES_PER_BLOCK + wave;
    if (bag >= n_bags) return;
    const int32_t t = (int32_t)(bag / B);
    const int32_t b = (int32_t)(bag - (int64_t)t * B);
    const float* __restrict__ tab = tables[t];
    const int64_t beg = off[bag];
    const int32_t L = (int32_t)(off[bag + 1] - beg);

    const int sub = lane / LPR;
    const int col = (lane % LPR) * 4;
    const bool col_ok = col < D;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);

    for (int32_t base = 0; base < L; base += REC_WAVE) {
        const int32_t n = min(REC_WAVE, L - base);
        const int32_t my_idx = (lane < n) ? indices[beg + base + lane] : 0;
        const int32_t groups = (n + RPI - 1) / RPI;
        for (int32_t g0 = 0; g0 < groups; g0 += U) {
            float4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int32_t r = (g0 + u) * RPI + sub;
                const int32_t idx = __shfl(my_idx, r & (REC_WAVE - 1));
                v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (r < n && col_ok)
                    v[u] = *reinterpret_cast<const float4*>(tab + (int64_t)idx * D + col);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                acc.x += v[u].x;
                acc.y += v[u].y;
                acc.z += v[u].z;
                acc.w += v[u].w;
            }
        }
    }
#pragma unroll
    for (int o = LPR; o < REC_WAVE; o <<= 1) {
        acc.x += __shfl_xor(acc.x, o);
        acc.y += __shfl_xor(acc.y, o);
        acc.z += __shfl_xor(acc.z, o);
        acc.w += __shfl_xor(acc.w, o);
    }
    if (sub == 0 && col_ok)
        *reinterpret_cast<float4*>(out + (int64_t)b * stride_b + (int64_t)t * stride_t + col) = acc;
}

// Bags of one or two lookups (the one-hot "Concat" models of Table I): a wavefront per bag
// would leave most lanes idle, so here each group of LPR lanes owns a bag of its own and a
// wavefront pools 64/LPR bags at once, rows added in index order.  Correct for any length;
// chosen by the host when the average bag is at most two lookups long.
template <int LPR>
__global__ __launch_bounds__(SLS_WAVES_PER_BLOCK* REC_WAVE) void sls_short_kernel(
    const float* const* __restrict__ tables, const int32_t* __restrict__ indices,
    const int64_t* __restrict__ off, int64_t n_bags, int32_t B, int32_t D, float* __restrict__ out,
    int64_t stride_b, int64_t stride_t) {
    constexpr int G = REC_WAVE / LPR;
    constexpr int U = 4;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane / LPR;
    const int col = (lane % LPR) * 4;
    const int64_t bag = ((int64_t)blockIdx.x * SLS_WAVES_PER_BLOCK + wave) * G + sub;
    if (bag >= n_bags || col >= D) return;              // no cross-lane traffic below
    const int32_t t = (int32_t)(bag / B);
    const int32_t b = (int32_t)(bag - (int64_t)t * B);
    const float* __restrict__ tab = tables[t];
    const int64_t beg = off[bag];
    const int32_t L = (int32_t)(off[bag + 1] - beg);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int32_t j = 0; j < L; j += U) {
        int32_t idx[U];
#pragma unroll
        for (int u = 0; u < U; ++u) idx[u] = (j + u < L) ? indices[beg + j + u] : -1;
        float4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (idx[u] >= 0) v[u] = *reinterpret_cast<const float4*>(tab + (int64_t)idx[u] * D + col);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            acc.x += v[u].x;
            acc.y += v[u].y;
            acc.z += v[u].z;
            acc.w += v[u].w;
        }
    }
    *reinterpret_cast<float4*>(out + (int64_t)b * stride_b + (int64_t)t * stride_t + col) = acc;
}

// ------------------------------------------------------------------ validator
// res[0] = sum of lengths, res[1] = 1 if any length < 0,
// res[2] = number of out-of-range indices, res[3] = position of the first one.
__global__ __launch_bounds__(256) void check_lengths_kernel(const int32_t* __restrict__ len, int64_t n,
                                                            unsigned long long* res) {
    int64_t s = 0;
    int neg = 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int32_t v = len[i];
        s += v;
        neg |= (v < 0);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        s += __shfl_xor(s, o);
        neg |= __shfl_xor(neg, o);
    }
    if ((threadIdx.x & 63) == 0) {
        atomicAdd(&res[0], (unsigned long long)s);
        if (neg) atomicOr(&res[1], 1ull);
    }
}

__global__ __launch_bounds__(256) void check_indices_kernel(const int32_t* __restrict__ indices,
                                                            const int64_t* __restrict__ off,
                                                            const int64_t* __restrict__ rows, int64_t n_bags,
                                                            int32_t B, unsigned long long* res) {
    const int lane = threadIdx.x & 63;
    const int64_t bag = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (bag >= n_bags) return;
    const int64_t R = rows[bag / B];
    const int64_t beg = off[bag], end = off[bag + 1];
    unsigned long long bad = 0, first = ~0ull;
    for (int64_t p = beg + lane; p < end; p += REC_WAVE) {
        const int64_t idx = indices[p];
        if (idx < 0 || idx >= R) {
            ++bad;
            if ((unsigned long long)p < first) first = (unsigned long long)p;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        bad += __shfl_xor(bad, o);
        const unsigned long long other = __shfl_xor(first, o);
        first = other < first ? other : first;
    }
    if (lane == 0 && bad) {
        atomicAdd(&res[2], bad);
        atomicMin(&res[3], first);
    }
}

struct SlsWorkspace {
    int64_t* offsets;
    unsigned long long* results;
    int64_t* rows;
};

size_t sls_offsets_bytes(int32_t T, int32_t B) {
    return rec_round_up(((size_t)T * (size_t)B + 1) * sizeof(int64_t), 256);
}

SlsWorkspace carve(void* ws, int32_t T, int32_t B) {
    char* p = static_cast<char*>(ws);
    SlsWorkspace w;
    w.offsets = reinterpret_cast<int64_t*>(p);
    p += sls_offsets_bytes(T, B);
    w.results = reinterpret_cast<unsigned long long*>(p);
    p += 256;
    w.rows = reinterpret_cast<int64_t*>(p);
    return w;
}

rec_status check_sparse_args(const int64_t* rows, int32_t T, const int32_t* indices, int64_t n_indices,
                             const int32_t* lengths, int32_t B) {
    if (T < 1 || B < 0 || n_indices < 0) return REC_ERR_BAD_SHAPE;
    if (!rows) return REC_ERR_NULL;
    if (B > 0 && !lengths) return REC_ERR_NULL;
    if (n_indices > 0 && !indices) return REC_ERR_NULL;
    for (int32_t t = 0; t < T; ++t) {
        if (rows[t] < 1) return REC_ERR_BAD_SHAPE;
        if (rows[t] > 2147483647LL) return REC_ERR_UNSUPPORTED;
    }
    return REC_OK;
}

rec_status launch_offsets(const int32_t* lengths, int64_t n_bags, int64_t* offsets, hipStream_t s) {
    const int tiles = rec_scan_parallel_tiles(n_bags);
    hipLaunchKernelGGL(offsets_kernel, dim3(tiles > 0 ? (unsigned)tiles : 1u), dim3(SCAN_THREADS), 0, s, lengths,
                       n_bags, offsets, (int)rec_aligned(lengths, 16));
    REC_CHECK_LAUNCH();
    return REC_OK;
}

}  // namespace

int rec_scan_parallel_tiles(int64_t n) {
    const int64_t tiles = (n + SCAN_TILE - 1) / SCAN_TILE;
    return (tiles >= 1 && tiles <= SCAN_MAX_PARALLEL_TILES) ? (int)tiles : 0;
}

rec_status rec_scan_launch(const rec_scan_job& job, hipStream_t s) {
    return launch_offsets(job.lengths, job.n, job.offsets, s);
}

int64_t* rec_sls_workspace_offsets(void* workspace) { return static_cast<int64_t*>(workspace); }

static rec_status rec_sls_launch(const float* const* tables, int32_t T, int32_t D, const int32_t* indices,
                          int64_t n_indices, const int64_t* offsets, int32_t B, float* out, int64_t stride_b,
                          int64_t stride_t, hipStream_t s) {
    const int64_t n_bags = (int64_t)T * B;
    if (n_indices <= 2 * n_bags) {
        // short bags: several bags per wavefront
#define SLS_SHORT(LPR)                                                                                        \
    do {                                                                                                      \
        const int64_t per_block = (int64_t)SLS_WAVES_PER_BLOCK * (REC_WAVE / LPR);                            \
        const int64_t blocks = (n_bags + per_block - 1) / per_block;                                          \
        hipLaunchKernelGGL((sls_short_kernel<LPR>), dim3((unsigned)blocks), dim3(SLS_WAVES_PER_BLOCK* REC_WAVE), 0, s, \
                           tables, indices, offsets, n_bags, B, D, out, stride_b, stride_t);                  \
    } while (0)
        if (D <= 16) SLS_SHORT(4);
        else if (D <= 32) SLS_SHORT(8);
        else if (D <= 64) SLS_SHORT(16);
        else if (D <= 128) SLS_SHORT(32);
        else SLS_SHORT(64);
#undef SLS_SHORT
        REC_CHECK_LAUNCH();
        return REC_OK;
    }
    const int64_t blocks = (n_bags + SLS_WAVES_PER_BLOCK - 1) / SLS_WAVES_PER_BLOCK;
    if (blocks > 2147483647LL) return REC_ERR_UNSUPPORTED;
    const dim3 grid((unsigned)blocks), block(SLS_WAVES_PER_BLOCK * REC_WAVE);
#define SLS_LAUNCH(LPR, U)                                                                            \
    hipLaunchKernelGGL((sls_kernel<LPR, U>), grid, block, 0, s, tables, indices, offsets, n_bags, B, D, \
                       out, stride_b, stride_t)
    // 8 row loads in flight per lane: 56 registers, 8 waves per SIMD.  Swept 4..32 on the 64-wide rows
    // of the embedding-dominated model: deeper unrolling costs occupancy (16 -> 100 registers, 4 waves)
    // and 15 % of the rate when rows hit in cache; with uniform indices every depth runs at the same,
    // memory-bound, speed.
    if (D <= 16) SLS_LAUNCH(4, 4);
    else if (D <= 32) SLS_LAUNCH(8, 8);
    else if (D <= 64) SLS_LAUNCH(16, 8);
    else if (D <= 128) SLS_LAUNCH(32, 8);
    else SLS_LAUNCH(64, 8);
#undef SLS_LAUNCH
    REC_CHECK_LAUNCH();
    return REC_OK;
}

extern "C" {

size_t rec_sls_workspace_bytes(int32_t T, int32_t B) {
    if (T < 1 || B < 0) return 0;
    return sls_offsets_bytes(T, B) + 256 + rec_round_up((size_t)T * sizeof(int64_t), 256);
}

rec_status rec_sls_offsets(const int32_t* lengths, int64_t n_bags, int64_t* offsets, void* stream) {
    if (n_bags < 0) return REC_ERR_BAD_SHAPE;
    if (!offsets || (n_bags > 0 && !lengths)) return REC_ERR_NULL;
    if (!rec_aligned(offsets, 8)) return REC_ERR_BAD_SHAPE;
    return launch_offsets(lengths, n_bags, offsets, static_cast<hipStream_t>(stream));
}

rec_status rec_sls_forward(const float* const* tables, const int64_t* rows, int32_t T, int32_t D,
                           const int32_t* indices, int64_t n_indices, const int32_t* lengths, int32_t B,
                           float* out, int64_t out_stride_b, int64_t out_stride_t, void* workspace,
                           size_t workspace_bytes, void* stream) {
    return rec_sls_forward_step(tables, rows, T, D, indices, n_indices, lengths, B, out, out_stride_b, out_stride_t,
                                workspace, workspace_bytes, stream, REC_SLS_ALL);
}

}  // extern "C"

// ---- pooling without a workspace argument -------------------------------------------------------
// The bag offsets of rec_sls_forward_static live in this array: one copy per GPU the library runs
// on, held until the process ends.  In host code the name is only a handle for
// hipGetSymbolAddress; kernels get the device address that call returns.
static __device__ __align__(256) unsigned char sls_static_scratch[REC_SLS_STATIC_MAX_BAGS * sizeof(int64_t) + 256];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex static_scratch_mutex;
void* static_scratch_ptr[MAX_DEVICES];          // device address of the array on each device, once looked up

// Device address of sls_static_scratch on the current device (looked up on the first call on that device).
rec_status static_scratch(void** ptr) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return REC_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(static_scratch_mutex);
    if (!static_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(sls_static_scratch)) != hipSuccess || !p) return REC_ERR_DEVICE;
        static_scratch_ptr[dev] = p;
    }
    *ptr = static_scratch_ptr[dev];
    return REC_OK;
}
}  // namespace

extern "C" rec_status rec_sls_forward_static(const float* const* tables, const int64_t* rows, int32_t T, int32_t D,
                                             const int32_t* indices, int64_t n_indices, const int32_t* lengths, int32_t B,
                                             float* out, int64_t out_stride_b, int64_t out_stride_t, void* stream) {
    rec_status st = check_sparse_args(rows, T, indices, n_indices, lengths, B);
    if (st != REC_OK) return st;
    if (!tables) return REC_ERR_NULL;
    if (D < 4 || D > 256 || D % 4) return REC_ERR_UNSUPPORTED;
    if ((int64_t)T * B + 1 > (int64_t)REC_SLS_STATIC_MAX_BAGS) return REC_ERR_WORKSPACE;   // more bags than the array holds
    if (B == 0) return REC_OK;
    if (!out) return REC_ERR_NULL;
    if (out_stride_b < 0 || out_stride_t < 0 || out_stride_b % 4 || out_stride_t % 4 || !rec_aligned(out, 16))
        return REC_ERR_BAD_SHAPE;
    void* scratch = nullptr;
    st = static_scratch(&scratch);
    if (st != REC_OK) return st;
    // every offset the pooling reads is written by the scan first, so nothing has to be cleared
    int64_t* offsets = static_cast<int64_t*>(scratch);
    hipStream_t s = static_cast<hipStream_t>(stream);
    st = launch_offsets(lengths, (int64_t)T * B, offsets, s);
    if (st != REC_OK) return st;
    return rec_sls_launch(tables, T, D, indices, n_indices, offsets, B, out, out_stride_b, out_stride_t, s);
}

rec_status rec_sls_forward_step(const float* const* tables, const int64_t* rows, int32_t T, int32_t D,
                                const int32_t* indices, int64_t n_indices, const int32_t* lengths, int32_t B, float* out,
                                int64_t out_stride_b, int64_t out_stride_t, void* workspace, size_t workspace_bytes,
                                void* stream, rec_sls_step step) {
    rec_status st = check_sparse_args(rows, T, indices, n_indices, lengths, B);
    if (st != REC_OK) return st;
    if (!tables) return REC_ERR_NULL;
    if (D < 4 || D > 256 || D % 4) return REC_ERR_UNSUPPORTED;
    if (B == 0) return REC_OK;
    if (!out) return REC_ERR_NULL;
    if (out_stride_b < 0 || out_stride_t < 0 || out_stride_b % 4 || out_stride_t % 4 || !rec_aligned(out, 16))
        return REC_ERR_BAD_SHAPE;
    if (!workspace || !rec_aligned(workspace, 256) || workspace_bytes < rec_sls_workspace_bytes(T, B))
        return REC_ERR_WORKSPACE;
    if (step == REC_SLS_CHECK_ONLY) return REC_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    SlsWorkspace w = carve(workspace, T, B);
    if (step == REC_SLS_ALL) {
        st = launch_offsets(lengths, (int64_t)T * B, w.offsets, s);
        if (st != REC_OK) return st;
    }
    return rec_sls_launch(tables, T, D, indices, n_indices, w.offsets, B, out, out_stride_b, out_stride_t, s);
}

extern "C" {

rec_status rec_sls_forward_offsets(const float* const* tables, const int64_t* rows, int32_t T, int32_t D,
                                   const int32_t* indices, int64_t n_indices, const int64_t* offsets, int32_t B,
                                   float* out, int64_t out_stride_b, int64_t out_stride_t, void* stream) {
    if (T < 1 || B < 0 || n_indices < 0) return REC_ERR_BAD_SHAPE;
    if (!rows || !tables) return REC_ERR_NULL;
    for (int32_t t = 0; t < T; ++t) {
        if (rows[t] < 1) return REC_ERR_BAD_SHAPE;
        if (rows[t] > 2147483647LL) return REC_ERR_UNSUPPORTED;
    }
    if (D < 4 || D > 256 || D % 4) return REC_ERR_UNSUPPORTED;
    if (B == 0) return REC_OK;
    if (!out || !offsets || (n_indices > 0 && !indices)) return REC_ERR_NULL;
    if (out_stride_b < 0 || out_stride_t < 0 || out_stride_b % 4 || out_stride_t % 4 || !rec_aligned(out, 16) ||
        !rec_aligned(offsets, 8))
        return REC_ERR_BAD_SHAPE;
    return rec_sls_launch(tables, T, D, indices, n_indices, offsets, B, out, out_stride_b, out_stride_t,
                          static_cast<hipStream_t>(stream));
}

rec_status rec_sls_validate(const int64_t* rows, int32_t T, const int32_t* indices, int64_t n_indices,
                            const int32_t* lengths, int32_t B, int64_t* n_bad, int64_t* first_bad,
                            void* workspace, size_t workspace_bytes, void* stream) {
    if (n_bad) *n_bad = 0;
    if (first_bad) *first_bad = -1;
    rec_status st = check_sparse_args(rows, T, indices, n_indices, lengths, B);
    if (st != REC_OK) return st;
    if (!workspace || !rec_aligned(workspace, 256) || workspace_bytes < rec_sls_workspace_bytes(T, B))
        return REC_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    SlsWorkspace w = carve(workspace, T, B);
    const int64_t n_bags = (int64_t)T * B;

    unsigned long long res[4] = {0ull, 0ull, 0ull, ~0ull};
    if (hipMemcpyAsync(w.results, res, sizeof(res), hipMemcpyHostToDevice, s) != hipSuccess) return REC_ERR_DEVICE;
    if (hipMemcpyAsync(w.rows, rows, (size_t)T * sizeof(int64_t), hipMemcpyHostToDevice, s) != hipSuccess)
        return REC_ERR_DEVICE;
    if (n_bags > 0) {
        const unsigned grid = (unsigned)((n_bags + 255) / 256 < 1024 ? (n_bags + 255) / 256 : 1024);
        hipLaunchKernelGGL(check_lengths_kernel, dim3(grid), dim3(256), 0, s, lengths, n_bags, w.results);
        REC_CHECK_LAUNCH();
    }
    if (hipMemcpyAsync(res, w.results, sizeof(res), hipMemcpyDeviceToHost, s) != hipSuccess) return REC_ERR_DEVICE;
    if (hipStreamSynchronize(s) != hipSuccess) return REC_ERR_DEVICE;
    if (res[1]) return REC_ERR_NEGATIVE_LENGTH;
    if ((int64_t)res[0] != n_indices) return REC_ERR_LENGTHS_MISMATCH;
    if (n_bags == 0 || n_indices == 0) return REC_OK;

    st = launch_offsets(lengths, n_bags, w.offsets, s);
    if (st != REC_OK) return st;
    const int64_t blocks = (n_bags + 3) / 4;
    if (blocks > 2147483647LL) return REC_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(check_indices_kernel, dim3((unsigned)blocks), dim3(256), 0, s, indices, w.offsets, w.rows,
                       n_bags, B, w.results);
    REC_CHECK_LAUNCH();
    if (hipMemcpyAsync(res, w.results, sizeof(res), hipMemcpyDeviceToHost, s) != hipSuccess) return REC_ERR_DEVICE;
    if (hipStreamSynchronize(s) != hipSuccess) return REC_ERR_DEVICE;
    if (res[2]) {
        if (n_bad) *n_bad = (int64_t)res[2];
        if (first_bad) *first_bad = (int64_t)res[3];
        return REC_ERR_INDEX_RANGE;
    }
    return REC_OK;
}

}  // extern "C"
