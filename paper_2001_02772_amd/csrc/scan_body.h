// Offsets scan over the bag lengths (off[0] = 0, off[i+1] = off[i] + len[i]): the block-level
// body, shared by the stand-alone scan launch and by launches that carry the scan next to
// other work.  Feeds the pooling of Section II-A (DeepRecSys paper): bags are given by their
// lengths, the kernel needs where each bag starts.
#ifndef REC_SCAN_BODY_H
#define REC_SCAN_BODY_H
#include "rec_common.h"

namespace {

// ------------------------------------------------------------------ offsets scan
constexpr int SCAN_THREADS = 1024;
constexpr int SCAN_ITEMS = 4;
constexpr int SCAN_TILE = SCAN_THREADS * SCAN_ITEMS;
constexpr int SCAN_MAX_PARALLEL_TILES = 64;

__device__ __forceinline__ int64_t wave_inclusive_scan(int64_t v, int lane) {
#pragma unroll
    for (int o = 1; o < REC_WAVE; o <<= 1) {
        int64_t up = __shfl_up(v, o);
        if (lane >= o) v += up;
    }
    return v;
}

// Block-wide exclusive scan of `v` (one value per thread) fused with a block-wide sum of
// `extra`: returns the exclusive prefix of v, leaves the block totals in *v_total and
// *extra_total.  smem holds two slots per wave.
__device__ __forceinline__ int64_t block_scan_and_sum(int64_t v, int64_t extra, int64_t* smem, int64_t* v_total,
                                                      int64_t* extra_total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n_waves = blockDim.x >> 6;
    const int64_t incl = wave_inclusive_scan(v, lane);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) extra += __shfl_xor(extra, o);
    __syncthreads();                       // smem may still be read from a previous call
    if (lane == 63) {
        smem[2 * wave] = incl;
        smem[2 * wave + 1] = extra;
    }
    __syncthreads();
    int64_t wave_base = 0, tot = 0, etot = 0;
    for (int w = 0; w < n_waves; ++w) {
        const int64_t s = smem[2 * w];
        if (w < wave) wave_base += s;
        tot += s;
        etot += smem[2 * w + 1];
    }
    *v_total = tot;
    *extra_total = etot;
    return wave_base + incl - v;
}

// off[0] = 0, off[i+1] = off[i] + len[i].
// A batch has a few tens of thousands of bags, so the scan is a latency chain, not a
// bandwidth problem.  gridDim.x > 1: block k owns tile k (4096 lengths) and re-adds every
// length before its tile with wide, independent loads (at most a few hundred KB, all in
// L2) -- one launch, no inter-block waiting; the tile's own loads are issued first so both
// latencies overlap, and one pass over LDS does the tile scan and the prefix sum together.
// otherwise (very long inputs): a single block walks the tiles in order carrying the
// running sum.
// `my_tile` / `parallel` select the mode, so that a launch which also carries other work can
// hand some of its blocks to the scan.
__device__ __forceinline__ void offsets_block(const int32_t* __restrict__ len, int64_t n, int64_t* __restrict__ off,
                                              int vec_ok, int my_tile, bool parallel) {
    __shared__ int64_t smem[2 * SCAN_THREADS / REC_WAVE];
    const int tid = threadIdx.x;
    int64_t carry = 0;
    const int64_t tile_begin = parallel ? my_tile : 0;
    const int64_t tile_end = parallel ? tile_begin + 1 : (n + SCAN_TILE - 1) / SCAN_TILE;
    for (int64_t tile = tile_begin; tile < tile_end; ++tile) {
        const int64_t first = tile * SCAN_TILE + (int64_t)tid * SCAN_ITEMS;
        int32_t v[SCAN_ITEMS];
        if (vec_ok && first + SCAN_ITEMS <= n) {
            const int4 q = *reinterpret_cast<const int4*>(len + first);
            v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
        } else {
#pragma unroll
            for (int k = 0; k < SCAN_ITEMS; ++k) v[k] = (first + k < n) ? len[first + k] : 0;
        }
        int64_t part = 0;
        if (parallel) {
            const int64_t before = tile_begin * SCAN_TILE;          // a multiple of 4
            if (vec_ok) {
                const int4* __restrict__ len4 = reinterpret_cast<const int4*>(len);
                const int64_t nv = before / 4;
                for (int64_t i = tid; i < nv; i += 16 * SCAN_THREADS) {
                    int4 q[16];
#pragma unroll
                    for (int k = 0; k < 16; ++k) {        // unconditional loads from clamped addresses
                        const int64_t j = i + k * SCAN_THREADS;
                        q[k] = len4[j < nv ? j : nv - 1];
                    }
#pragma unroll
                    for (int k = 0; k < 16; ++k)
                        if (i + k * SCAN_THREADS < nv) part += (int64_t)q[k].x + q[k].y + q[k].z + q[k].w;
                }
            } else {
                for (int64_t i = tid; i < before; i += 8 * SCAN_THREADS) {
                    int32_t q[8];
#pragma unroll
                    for (int k = 0; k < 8; ++k)
                        q[k] = (i + k * SCAN_THREADS < before) ? len[i + k * SCAN_THREADS] : 0;
#pragma unroll
                    for (int k = 0; k < 8; ++k) part += q[k];
                }
            }
        }
        int64_t s = 0;
#pragma unroll
        for (int k = 0; k < SCAN_ITEMS; ++k) s += v[k];
        int64_t tot, before_tot;
        int64_t run = block_scan_and_sum(s, part, smem, &tot, &before_tot) + carry + before_tot;
        int64_t o[SCAN_ITEMS];
#pragma unroll
        for (int k = 0; k < SCAN_ITEMS; ++k) {
            run += v[k];
            o[k] = run;
        }
#pragma unroll
        for (int k = 0; k < SCAN_ITEMS; ++k)
            if (first + k < n) off[first + k + 1] = o[k];
        carry += tot;
    }
    if (my_tile == 0 && tid == 0) off[0] = 0;
}

}  // namespace

#endif
