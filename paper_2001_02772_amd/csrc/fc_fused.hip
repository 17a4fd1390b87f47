// Several narrow FC layers in one launch.
//
// The Dense-FC and Predict-FC stacks of Table I (DeepRecSys paper, Section II-A)
// end in -- or consist of -- layers a few hundred units wide.  At a batch of a
// thousand rows each such layer is a few microseconds of matrix-core work, so a
// launch per layer is mostly launch latency and a round trip of the activations
// through memory.  Here a block takes 16 samples through up to four consecutive
// layers: activations stay in LDS (two ping-pong buffers), the weights of each
// layer stream from L2 straight into MFMA operand registers (every block reads
// them once), and only the last layer's output goes back to memory.
// fp32: v_mfma_f32_16x16x4_f32;  bf16 operands: v_mfma_f32_16x16x32_bf16.
#include "rec_common.h"
#include "scan_body.h"

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short ushort8 __attribute__((ext_vector_type(8)));

constexpr int FM_ROWS = 16;
constexpr int FM_WAVES = 16;
constexpr int FM_THREADS = FM_WAVES * 64;

// Interaction computed in the block (see rec_fused_mlp_args::vecs): a sample's V vectors are kept
// in LDS with a row stride of D + 1 floats (odd, so the rows of different vectors fall into
// different banks), at most FI_SAMPLE floats per sample and FI_PAIRS pairs.
constexpr int FI_SAMPLE = 1024;
constexpr int FI_PAIRS = 1024;

template <bool BF16>
struct FM {
    static constexpr int MAXW = BF16 ? REC_FUSED_MAX_WIDTH_BF16 : REC_FUSED_MAX_WIDTH_F32;
    static constexpr int ELT = BF16 ? 2 : 4;
    static constexpr int KCH = BF16 ? 32 : 16;                 // k covered by one operand load per lane
    static constexpr int LDA = MAXW + 16 / ELT;                // padded activation row (elements)
    static constexpr int BUF_BYTES = FM_ROWS * LDA * ELT;
    typedef typename std::conditional<BF16, uint16_t, float>::type act_t;
};

template <bool BF16>
__device__ __forceinline__ typename FM<BF16>::act_t to_act(float v) {
    if constexpr (BF16) return rec_f32_to_bf16_bits(v);
    else return v;
}

// One pipeline item: the weights a lane needs for GU consecutive k-chunks of one 16-column tile.
template <bool BF16>
struct WGroup {
    static constexpr int GU = 4;
    typedef typename std::conditional<BF16, ushort8, float4>::type reg_t;
    reg_t w[GU];
    float bias;          // bias of output column n0 + (lane % 16): fetched with the weights so that the
                         // tile's epilogue never waits for a load of its own
};

// Raw loads of one item: lane (li, q) fetches, for each of the GU chunks, the VEC consecutive k
// of weight row n0+li that it will feed to the MFMAs.  Out-of-range lanes read a valid (clamped)
// address and the value is discarded by mask_group() when the item is consumed.  Nothing here
// uses a loaded value, so the loads stay in flight while the previous item is multiplied.
template <bool BF16>
__device__ __forceinline__ void load_group(WGroup<BF16>& g, const void* Wv, const float* __restrict__ bias, int K, int N,
                                           int n0, int k0, int li, int q) {
    constexpr int KCH = FM<BF16>::KCH;
    constexpr int VEC = BF16 ? 8 : 4;
    typedef typename std::conditional<BF16, uint16_t, float>::type w_t;
    typedef typename WGroup<BF16>::reg_t reg_t;
    const w_t* __restrict__ W = static_cast<const w_t*>(Wv);
    const bool vec = (K % VEC == 0) && rec_dev_aligned(W, 16);
    const int n = n0 + li;
    const w_t* wrow = W + (int64_t)(n < N ? n : 0) * K;
    g.bias = bias[n < N ? n : 0];
    if (vec) {
#pragma unroll
        for (int u = 0; u < WGroup<BF16>::GU; ++u) {
            const int kk = k0 + KCH * u + VEC * q;
            g.w[u] = *reinterpret_cast<const reg_t*>(wrow + (kk < K ? kk : 0));
        }
    } else {
#pragma unroll
        for (int u = 0; u < WGroup<BF16>::GU; ++u) {
            const int kk = k0 + KCH * u + VEC * q;
            reg_t v;
            if constexpr (BF16) v = ushort8{0, 0, 0, 0, 0, 0, 0, 0};
            else v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (k0 + KCH * u < K) {                       // wave-uniform: skip chunks wholly past K
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const w_t t = wrow[kk + e < K ? kk + e : 0];
                    if constexpr (BF16) v[e] = t;
                    else (&v.x)[e] = t;
                }
            }
            g.w[u] = v;
        }
    }
}

// Zero the weights that lie outside [N x K] (see load_group).
template <bool BF16>
__device__ __forceinline__ void mask_group(WGroup<BF16>& g, int K, int N, int n, int k0, int q) {
    constexpr int KCH = FM<BF16>::KCH;
    constexpr int VEC = BF16 ? 8 : 4;
#pragma unroll
    for (int u = 0; u < WGroup<BF16>::GU; ++u) {
        const int kk = k0 + KCH * u + VEC * q;
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const bool ok = n < N && kk + e < K;
            if constexpr (BF16) g.w[u][e] = ok ? g.w[u][e] : (unsigned short)0;
            else (&g.w[u].x)[e] = ok ? (&g.w[u].x)[e] : 0.f;
        }
    }
}

template <bool BF16>
__device__ __forceinline__ void mfma_chunk(floatx4& acc, const typename FM<BF16>::act_t* xrow, int k,
                                           const typename WGroup<BF16>::reg_t& w) {
    if constexpr (!BF16) {
        // lane (row, q) feeds k = 4q..4q+3 of each 16-chunk to four MFMAs, one component each; x and
        // W use the same assignment, so every k is multiplied exactly once
        const float4 x = *reinterpret_cast<const float4*>(xrow + k);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(x.x, w.x, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(x.y, w.y, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(x.z, w.z, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(x.w, w.w, acc, 0, 0, 0);
    } else {
        const ushort8 xs = *reinterpret_cast<const ushort8*>(xrow + k);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, xs), __builtin_bit_cast(bf16x8, w), acc,
                                                       0, 0, 0);
    }
}

// The layer table of the kernel arguments, copied once into scalar registers.  Lookups by a
// (wave-uniform) run-time layer number are chains of scalar selects instead of dependent loads
// from the argument buffer.
struct LayerTab {
    int w0, w1, w2, w3, w4;
    const void *W0, *W1, *W2, *W3;
    const float *b0, *b1, *b2, *b3;
    int a0, a1, a2, a3;
    int n_layers;

    __device__ __forceinline__ explicit LayerTab(const rec_fused_mlp_args& a)
        : w0(a.width[0]), w1(a.width[1]), w2(a.width[2]), w3(a.width[3]), w4(a.width[4]),
          W0(a.W[0]), W1(a.W[1]), W2(a.W[2]), W3(a.W[3]),
          b0(a.bias[0]), b1(a.bias[1]), b2(a.bias[2]), b3(a.bias[3]),
          a0(a.act[0]), a1(a.act[1]), a2(a.act[2]), a3(a.act[3]), n_layers(a.n_layers) {
        static_assert(REC_FUSED_MAX_LAYERS == 4, "LayerTab is written out for four layers");
    }
    __device__ __forceinline__ int w(int i) const { return i == 0 ? w0 : i == 1 ? w1 : i == 2 ? w2 : i == 3 ? w3 : w4; }
    __device__ __forceinline__ const void* wt(int l) const { return l == 0 ? W0 : l == 1 ? W1 : l == 2 ? W2 : W3; }
    __device__ __forceinline__ const float* b(int l) const { return l == 0 ? b0 : l == 1 ? b1 : l == 2 ? b2 : b3; }
    __device__ __forceinline__ int ac(int l) const { return l == 0 ? a0 : l == 1 ? a1 : l == 2 ? a2 : a3; }
};

// What one wave does in one layer.  A layer has Np/16 column tiles.  With at least 16 tiles
// wave w takes tiles w, w+16, ... over the whole of k.  With fewer, the spare waves split k:
// ks waves share a tile, each taking a contiguous run of k-groups, and their partial tiles are
// folded through LDS in wave order (fixed, so results are reproducible).  All fields are
// wave-uniform.
struct WavePlan {
    int n_first, n_step, n_end;   // column tiles: n0 = n_first, n_first + n_step, ... < n_end
    int k_begin, k_end;           // k-groups: k0 = k_begin, k_begin + GK, ... < k_end
    int ks, kpart, pass_waves;    // split factor, this wave's part, waves per k-part
    int parts;                    // k-parts that actually hold k-groups (<= ks)
};

template <bool BF16>
__device__ __forceinline__ WavePlan plan_layer(const LayerTab& t, int l, int wave) {
    constexpr int KCH = FM<BF16>::KCH;
    constexpr int GK = KCH * WGroup<BF16>::GU;
    const int Kp = (t.w(l) + KCH - 1) / KCH * KCH;
    const int Np = (t.w(l + 1) + KCH - 1) / KCH * KCH;
    const int tiles = Np / 16, groups = (Kp + GK - 1) / GK;
    int ks = 1;
    while (ks * 2 * tiles <= FM_WAVES && ks * 2 <= groups) ks *= 2;
    WavePlan p;
    p.ks = ks;
    p.pass_waves = FM_WAVES / ks;
    p.kpart = wave / p.pass_waves;
    const int gper = (groups + ks - 1) / ks;
    p.parts = (groups + gper - 1) / gper;
    p.k_begin = p.kpart * gper * GK;
    p.k_end = (p.k_begin + gper * GK < Kp) ? p.k_begin + gper * GK : Kp;
    p.n_first = (wave % p.pass_waves) * 16;
    p.n_step = p.pass_waves * 16;
    p.n_end = (p.k_begin < p.k_end) ? Np : 0;
    return p;
}

// Position of a wave in its work list: layer, column tile, k-group.
struct Cursor {
    int l, n0, k0;
    WavePlan p;
};

// First item of layer c.l or of the next layer in which the wave has work; false if none.
template <bool BF16>
__device__ __forceinline__ bool cursor_enter(Cursor& c, const LayerTab& t, int wave) {
    while (c.l < t.n_layers) {
        c.p = plan_layer<BF16>(t, c.l, wave);
        if (c.p.n_first < c.p.n_end) {
            c.n0 = c.p.n_first;
            c.k0 = c.p.k_begin;
            return true;
        }
        ++c.l;
    }
    return false;
}

template <bool BF16>
__device__ __forceinline__ bool cursor_next(Cursor& c, const LayerTab& t, int wave) {
    constexpr int GK = FM<BF16>::KCH * WGroup<BF16>::GU;
    c.k0 += GK;
    if (c.k0 < c.p.k_end) return true;
    c.k0 = c.p.k_begin;
    c.n0 += c.p.n_step;
    if (c.n0 < c.p.n_end) return true;
    ++c.l;
    return cursor_enter<BF16>(c, t, wave);
}

// Issue the loads of the item the cursor points at.
template <bool BF16>
__device__ __forceinline__ void fetch_item(WGroup<BF16>& g, const Cursor& c, const LayerTab& t, int li, int q) {
    load_group<BF16>(g, t.wt(c.l), t.b(c.l), t.w(c.l), t.w(c.l + 1), c.n0, c.k0, li, q);
}

// Bias, activation and store of one 16x16 tile.  MFMA 16x16 accumulator layout: register v of
// lane l holds row 4*(l/16)+v, column l%16.  Hidden layers go to the LDS buffer of the next layer
// (columns past N are written as zeros: they are that layer's k padding), the last one to memory.
template <bool BF16>
__device__ __forceinline__ void tile_out(const floatx4& acc, int n, int N, int q, float bias, int act,
                                         bool last, typename FM<BF16>::act_t* out, const rec_fused_mlp_args& a, int m0) {
    const float bv = (n < N) ? bias : 0.f;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int r = 4 * q + v;
        const float z = (n < N) ? rec_apply_act(acc[v] + bv, act) : 0.f;
        if (!last) {
            out[r * FM<BF16>::LDA + n] = to_act<BF16>(z);
        } else if (n < N && m0 + r < a.B) {
            if (a.y_bf16) static_cast<uint16_t*>(a.y)[(int64_t)(m0 + r) * a.ldy + n] = rec_f32_to_bf16_bits(z);
            else static_cast<float*>(a.y)[(int64_t)(m0 + r) * a.ldy + n] = z;
        }
    }
}

// Weights do not depend on activations, so a wave always has the weights (and the bias) of its
// NEXT item in flight -- across column tiles and across layer boundaries -- while it multiplies
// the current one; the only exposed latencies are the first load and the input rows.  What bounds
// a block is the bytes it keeps in flight, so all 16 waves are given weight rows to fetch.
// (Three items ahead instead of one measured slower: 15.7 -> 18.9 us for 512-128-1 in fp32.)
template <bool BF16, bool INTER>
__device__ __forceinline__ void fused_mlp_block(const rec_fused_mlp_args& a, const int block) {
    typedef FM<BF16> C;
    typedef typename C::act_t act_t;
    constexpr int KCH = C::KCH;
    constexpr int GU = WGroup<BF16>::GU;
    constexpr int GK = KCH * GU;
    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * C::BUF_BYTES];
    __shared__ float red[FM_WAVES * 4 * 64];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m0 = block * FM_ROWS;
    const int li = lane & 15, q = lane >> 4;
    const LayerTab t(a);

    Cursor nxt;
    nxt.l = 0;
    bool have_next = cursor_enter<BF16>(nxt, t, wave);
    WGroup<BF16> gn;
    if (have_next) fetch_item<BF16>(gn, nxt, t, li, q);

    // stage the 16 input rows, zero-padded to a whole number of k-chunks.  The loads of a round
    // are independent and issued together (wide ones when the rows allow), so the whole tile
    // costs about one memory latency.
    if constexpr (INTER) {
        // Pairwise-dot interaction of the block's 16 samples, straight into the first layer's input
        // buffer (Section II-A, "Feature Interaction"): every thread takes (sample, output column)
        // pairs; a column is either a copy of the dense vector or one dot product of D terms.
        __shared__ float vs[FM_ROWS * FI_SAMPLE];
        __shared__ unsigned char pair_i[FI_PAIRS], pair_j[FI_PAIRS];
        act_t* buf = reinterpret_cast<act_t*>(lds);
        const int V = a.V, D = a.D, ldv = D + 1, P = V * (V - 1) / 2, width = D + P;
        const int K0p = (t.w0 + KCH - 1) / KCH * KCH;
        const int per_sample = V * D;
        const float* __restrict__ src = a.vecs + (int64_t)m0 * per_sample;
        const int rows = (a.B - m0 < FM_ROWS) ? a.B - m0 : FM_ROWS;
        for (int e0 = 0; e0 < FM_ROWS * per_sample; e0 += 4 * FM_THREADS) {
            float v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int e = e0 + i * FM_THREADS + tid;
                const bool ok = e < rows * per_sample;
                v[i] = src[ok ? e : 0];
                if (!ok) v[i] = 0.f;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int e = e0 + i * FM_THREADS + tid;
                if (e < FM_ROWS * per_sample) {
                    const int s = e / per_sample, r = e - s * per_sample;
                    vs[s * FI_SAMPLE + (r / D) * ldv + r % D] = v[i];
                }
            }
        }
        for (int p = tid; p < P; p += FM_THREADS) {
            int i = 1;
            while ((i + 1) * i / 2 <= p) ++i;
            pair_i[p] = (unsigned char)i;
            pair_j[p] = (unsigned char)(p - i * (i - 1) / 2);
        }
        __syncthreads();
        for (int c = tid; c < FM_ROWS * K0p; c += FM_THREADS) {
            const int s = c / K0p, col = c - s * K0p;
            const float* __restrict__ sv = vs + s * FI_SAMPLE;
            float val = 0.f;
            if (col < D) {
                val = sv[col];
            } else if (col < width) {
                const float* __restrict__ vi = sv + pair_i[col - D] * ldv;
                const float* __restrict__ vj = sv + pair_j[col - D] * ldv;
                for (int d = 0; d < D; ++d) val = fmaf(vi[d], vj[d], val);
            }
            buf[s * C::LDA + col] = to_act<BF16>(val);
        }
    } else {
        act_t* buf = reinterpret_cast<act_t*>(lds);
        const int K0 = t.w0;
        const int K0p = (K0 + KCH - 1) / KCH * KCH;
        const bool rows16 = rec_dev_aligned(a.x, 16);
        if (!a.x_bf16 && K0 % 4 == 0 && a.ldx % 4 == 0 && rows16) {
            const float* __restrict__ x = static_cast<const float*>(a.x);
            const int per_row = K0p / 4, total = FM_ROWS * per_row;
            for (int e0 = 0; e0 < total; e0 += 4 * FM_THREADS) {
                float4 v[4];
                int r[4], c[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int e = e0 + i * FM_THREADS + tid;
                    r[i] = e / per_row;
                    c[i] = (e - r[i] * per_row) * 4;
                    const bool ok = e < total && m0 + r[i] < a.B && c[i] < K0;
                    v[i] = *reinterpret_cast<const float4*>(x + (ok ? (int64_t)(m0 + r[i]) * a.ldx + c[i] : 0));
                    if (!ok) v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (e0 + i * FM_THREADS + tid < total) {
                        act_t* d = buf + r[i] * C::LDA + c[i];
                        d[0] = to_act<BF16>(v[i].x);
                        d[1] = to_act<BF16>(v[i].y);
                        d[2] = to_act<BF16>(v[i].z);
                        d[3] = to_act<BF16>(v[i].w);
                    }
                }
            }
        } else if (BF16 && a.x_bf16 && K0 % 8 == 0 && a.ldx % 8 == 0 && rows16) {
            const uint16_t* __restrict__ x = static_cast<const uint16_t*>(a.x);
            const int per_row = K0p / 8, total = FM_ROWS * per_row;
            for (int e0 = 0; e0 < total; e0 += 4 * FM_THREADS) {
                ushort8 v[4];
                int r[4], c[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int e = e0 + i * FM_THREADS + tid;
                    r[i] = e / per_row;
                    c[i] = (e - r[i] * per_row) * 8;
                    const bool ok = e < total && m0 + r[i] < a.B && c[i] < K0;
                    v[i] = *reinterpret_cast<const ushort8*>(x + (ok ? (int64_t)(m0 + r[i]) * a.ldx + c[i] : 0));
                    if (!ok) v[i] = ushort8{0, 0, 0, 0, 0, 0, 0, 0};
                }
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (e0 + i * FM_THREADS + tid < total)
                        *reinterpret_cast<ushort8*>(reinterpret_cast<uint16_t*>(buf) + r[i] * C::LDA + c[i]) = v[i];
            }
        } else {
            const int total = FM_ROWS * K0p;
            for (int e0 = 0; e0 < total; e0 += 4 * FM_THREADS) {
                float v[4];
                int r[4], c[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int e = e0 + i * FM_THREADS + tid;
                    r[i] = e / K0p;
                    c[i] = e - r[i] * K0p;
                    const bool ok = e < total && m0 + r[i] < a.B && c[i] < K0;
                    const int64_t off = ok ? (int64_t)(m0 + r[i]) * a.ldx + c[i] : 0;
                    float xv;
                    if (a.x_bf16) xv = __uint_as_float((uint32_t) static_cast<const uint16_t*>(a.x)[off] << 16);
                    else xv = static_cast<const float*>(a.x)[off];
                    v[i] = ok ? xv : 0.f;
                }
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (e0 + i * FM_THREADS + tid < total) buf[r[i] * C::LDA + c[i]] = to_act<BF16>(v[i]);
            }
        }
    }
    __syncthreads();

    for (int l = 0; l < t.n_layers; ++l) {
        const int K = t.w(l), N = t.w(l + 1);
        const bool last = (l == t.n_layers - 1);
        const int act = t.ac(l);
        const act_t* in = reinterpret_cast<const act_t*>(lds + (l & 1) * C::BUF_BYTES);
        act_t* out = reinterpret_cast<act_t*>(lds + ((l + 1) & 1) * C::BUF_BYTES);
        const act_t* xrow = in + li * C::LDA + (BF16 ? 8 : 4) * q;
        const WavePlan p = plan_layer<BF16>(t, l, wave);

        // With ks > 1 a wave owns at most one (tile, k-part), so the tile loop runs at most once
        // and `acc` still holds that partial tile after it.
        floatx4 acc = {0.f, 0.f, 0.f, 0.f};
        float bv = 0.f;                                  // bias of the tile in hand (every item of a tile carries it)
        for (int n0 = p.n_first; n0 < p.n_end; n0 += p.n_step) {
            const int n = n0 + li;
            acc = floatx4{0.f, 0.f, 0.f, 0.f};
            for (int k0 = p.k_begin; k0 < p.k_end; k0 += GK) {
                WGroup<BF16> g = gn;                             // item (l, n0, k0)
                bv = g.bias;
                have_next = cursor_next<BF16>(nxt, t, wave);
                if (have_next) fetch_item<BF16>(gn, nxt, t, li, q);
                // only a tile on the edge of W holds lanes to discard
                if (n0 + 16 > N || k0 + GK > K) mask_group<BF16>(g, K, N, n, k0, q);
                if (k0 + GK <= p.k_end) {
#pragma unroll
                    for (int u = 0; u < GU; ++u) mfma_chunk<BF16>(acc, xrow, k0 + KCH * u, g.w[u]);
                } else {
#pragma unroll
                    for (int u = 0; u < GU; ++u)
                        if (k0 + KCH * u < p.k_end) mfma_chunk<BF16>(acc, xrow, k0 + KCH * u, g.w[u]);
                }
            }
            if (p.ks == 1) tile_out<BF16>(acc, n0 + li, N, q, bv, act, last, out, a, m0);
        }
        if (p.ks > 1) {
            const bool active = p.n_first < p.n_end;
            if (active && p.kpart > 0) {
#pragma unroll
                for (int v = 0; v < 4; ++v) red[(wave * 4 + v) * 64 + lane] = acc[v];
            }
            __syncthreads();
            if (active && p.kpart == 0) {
                for (int s2 = 1; s2 < p.parts; ++s2) {
                    const int w2 = wave + s2 * p.pass_waves;
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[v] += red[(w2 * 4 + v) * 64 + lane];
                }
                tile_out<BF16>(acc, p.n_first + li, N, q, bv, act, last, out, a, m0);
            }
        }
        __syncthreads();
    }
}

template <bool BF16, bool INTER>
__global__ __launch_bounds__(FM_THREADS) void fused_mlp_kernel(rec_fused_mlp_args a) {
    fused_mlp_block<BF16, INTER>(a, (int)blockIdx.x);
}

// The same stack with the bag-offsets scan in the first `scan_tiles` blocks of the launch: the
// scan is a handful of latency-bound blocks that the pooling kernel waits for, and this stack is
// what runs next to it on an otherwise idle device, so the two share one launch.  The scan
// blocks come first because the last tile has the longest prefix to re-add.
static_assert(FM_THREADS == SCAN_THREADS, "both roles use the same block size");
template <bool BF16>
__global__ __launch_bounds__(FM_THREADS) void fused_mlp_scan_kernel(rec_fused_mlp_args a, const int32_t* __restrict__ len,
                                                                    int64_t n, int64_t* __restrict__ off, int vec_ok,
                                                                    int scan_tiles) {
    if ((int)blockIdx.x < scan_tiles) offsets_block(len, n, off, vec_ok, (int)blockIdx.x, true);
    else fused_mlp_block<BF16, false>(a, (int)blockIdx.x - scan_tiles);
}

}  // namespace

bool rec_fused_interact_ok(int32_t V, int32_t D) {
    // LDS space per sample, the pair table (indices fit a byte), and the time the dots take at 16 samples a block
    return V >= 1 && V <= 255 && D >= 1 && (int64_t)V * (D + 1) <= FI_SAMPLE && (int64_t)V * (V - 1) / 2 <= FI_PAIRS &&
           (int64_t)V * V * D <= 8192;
}

rec_status rec_fused_mlp_launch(const rec_fused_mlp_args& a, rec_dtype dt, const rec_scan_job* scan, hipStream_t s) {
    const unsigned blocks = (unsigned)((a.B + FM_ROWS - 1) / FM_ROWS);
    if (a.vecs) {
        if (scan || !rec_fused_interact_ok(a.V, a.D) || a.width[0] < a.D + a.V * (a.V - 1) / 2) return REC_ERR_BAD_SHAPE;
        if (dt == REC_BF16)
            hipLaunchKernelGGL((fused_mlp_kernel<true, true>), dim3(blocks), dim3(FM_THREADS), 0, s, a);
        else
            hipLaunchKernelGGL((fused_mlp_kernel<false, true>), dim3(blocks), dim3(FM_THREADS), 0, s, a);
    } else if (scan) {
        const int tiles = rec_scan_parallel_tiles(scan->n);
        if (tiles < 1 || !scan->lengths || !scan->offsets) return REC_ERR_BAD_SHAPE;
        const int vec_ok = (int)rec_aligned(scan->lengths, 16);
        if (dt == REC_BF16)
            hipLaunchKernelGGL(fused_mlp_scan_kernel<true>, dim3(blocks + tiles), dim3(FM_THREADS), 0, s, a, scan->lengths,
                               scan->n, scan->offsets, vec_ok, tiles);
        else
            hipLaunchKernelGGL(fused_mlp_scan_kernel<false>, dim3(blocks + tiles), dim3(FM_THREADS), 0, s, a, scan->lengths,
                               scan->n, scan->offsets, vec_ok, tiles);
    } else if (dt == REC_BF16) {
        hipLaunchKernelGGL((fused_mlp_kernel<true, false>), dim3(blocks), dim3(FM_THREADS), 0, s, a);
    } else {
        hipLaunchKernelGGL((fused_mlp_kernel<false, false>), dim3(blocks), dim3(FM_THREADS), 0, s, a);
    }
    REC_CHECK_LAUNCH();
    return REC_OK;
}
