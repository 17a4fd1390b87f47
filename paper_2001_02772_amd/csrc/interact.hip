// Pairwise-dot feature interaction with strict-lower-triangle packing.
//
// Section II-A ("Feature Interaction") of the DeepRecSys paper: the dense-stack
// output and the pooled embeddings are combined before the predictor stack.
// Here the combination is the DLRM one: all pairwise dot products of the V = T+1
// vectors of a sample, the strict lower triangle packed row by row behind a copy
// of the dense vector.  Per sample this is a V x D matrix times its transpose
// with V and D in the tens.  The data moved ([B][V][D] in, [B][D+P] out) is
// small, but with plain FMAs every pair re-reads two rows from LDS, and LDS
// bandwidth then dominates; so the per-sample Gram matrix is computed by one
// pair of wavefronts on the fp32 matrix cores (v_mfma_f32_16x16x4_f32: true fp32
// products and sums), 16x16 tiles of the lower triangle only, and the strict
// lower triangle is packed on the way out.
#include "rec_common.h"

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int IT_THREADS = 256;

// SPB samples per block of 4 waves, so 4/SPB waves share a sample: they stage its V x D tile into
// LDS together (zero-padded to Vp x Dp, Vp = V rounded up to 16, Dp = D rounded up to 16) and
// split the 16x16 tiles of the lower triangle (ti >= tj) between them round-robin.
template <int SPB>
__global__ __launch_bounds__(IT_THREADS) void interact_mfma_kernel(const float* __restrict__ vecs, int32_t B, int32_t V,
                                                                   int32_t D, float* __restrict__ out, int64_t ldo,
                                                                   int32_t zero_to) {
    extern __shared__ __attribute__((aligned(16))) float sm[];
    constexpr int WPS = 4 / SPB;                       // waves per sample
    constexpr int TPS = WPS * 64;                      // threads per sample
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int slot = wave / WPS, wsub = wave % WPS, tsub = tid - slot * TPS;
    const int Vp = (V + 15) / 16 * 16, Dp = (D + 15) / 16 * 16, ldv = Dp + 4;
    const int64_t b = (int64_t)blockIdx.x * SPB + slot;
    const bool active = b < B;
    float* my = sm + slot * Vp * ldv;
    const float* __restrict__ v = vecs + (active ? b : 0) * (int64_t)V * D;
    float* __restrict__ o = out + (active ? b : 0) * ldo;

    // stage; eight independent 16-byte loads per thread per round
    const int q_per_row = Dp / 4, total = Vp * q_per_row;
    for (int f0 = 0; f0 < total; f0 += 8 * TPS) {
        float4 t[8];
        int r[8], c[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int f = f0 + i * TPS + tsub;
            r[i] = f / q_per_row;
            c[i] = (f - r[i] * q_per_row) * 4;
            const bool ok = f < total && r[i] < V && c[i] < D;
            t[i] = *reinterpret_cast<const float4*>(v + (ok ? r[i] * D + c[i] : 0));
            if (!ok) t[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (f0 + i * TPS + tsub < total) *reinterpret_cast<float4*>(&my[r[i] * ldv + c[i]]) = t[i];
    }
    __syncthreads();
    if (!active) return;
    for (int d = tsub; d < D; d += TPS) o[d] = my[d];
    // columns behind the packed triangle that the consumer reads as padding of its k range
    for (int c = D + V * (V - 1) / 2 + tsub; c < zero_to; c += TPS) o[c] = 0.f;

    // Z = V V^T on 16x16 tiles.  Lane (row l%16, q = l/16) owns k = 4q..4q+3 of each 16-wide k chunk
    // and feeds them to 4 MFMAs, one component each; both operands use the same k assignment.
    // Accumulator layout: register e of lane l holds row 4*(l/16) + e, column l%16.
    const int nt = Vp / 16;
    const int frag = (lane & 15) * ldv + (lane >> 4) * 4;
    int t_index = 0;
    for (int ti = 0; ti < nt; ++ti) {
        for (int tj = 0; tj <= ti; ++tj, ++t_index) {
            if (t_index % WPS != wsub) continue;
            floatx4 acc = {0.f, 0.f, 0.f, 0.f};
            const float* pa = my + ti * 16 * ldv + frag;
            const float* pb = my + tj * 16 * ldv + frag;
            for (int k = 0; k < Dp; k += 16) {
                const float4 a = *reinterpret_cast<const float4*>(pa + k);
                const float4 c = *reinterpret_cast<const float4*>(pb + k);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.x, c.x, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.y, c.y, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.z, c.z, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.w, c.w, acc, 0, 0, 0);
            }
            const int j = tj * 16 + (lane & 15);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int i = ti * 16 + 4 * (lane >> 4) + e;
                if (i < V && j < i) o[D + i * (i - 1) / 2 + j] = acc[e];
            }
        }
    }
}

}  // namespace

extern "C" rec_status rec_interact(const float* vecs, int32_t B, int32_t V, int32_t D, float* out, int64_t ldo,
                                   void* stream) {
    return rec_interact_padded(vecs, B, V, D, out, ldo, 0, stream);
}

rec_status rec_interact_padded(const float* vecs, int32_t B, int32_t V, int32_t D, float* out, int64_t ldo,
                               int32_t zero_to, void* stream) {
    if (B < 0 || V < 1) return REC_ERR_BAD_SHAPE;
    if (zero_to > ldo) return REC_ERR_BAD_SHAPE;
    if (V > 128 || D < 4 || D > 256 || D % 4) return REC_ERR_UNSUPPORTED;   // bounds the LDS tile at 130 KB
    if (ldo < (int64_t)D + (int64_t)V * (V - 1) / 2) return REC_ERR_BAD_SHAPE;
    if (B == 0) return REC_OK;
    if (!vecs || !out) return REC_ERR_NULL;
    if (!rec_aligned(vecs, 16)) return REC_ERR_BAD_SHAPE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t per_sample = (size_t)((V + 15) / 16 * 16) * ((D + 15) / 16 * 16 + 4) * sizeof(float);
    const size_t budget = 64 * 1024;
    if (2 * per_sample <= budget) {
        hipLaunchKernelGGL(interact_mfma_kernel<2>, dim3((unsigned)((B + 1) / 2)), dim3(IT_THREADS), 2 * per_sample, s, vecs,
                           B, V, D, out, ldo, zero_to);
    } else {
        // up to 128 x 260 floats = 130 KB for the largest supported shape: needs the opt-in above 64 KB
        static const hipError_t big_lds = hipFuncSetAttribute(reinterpret_cast<const void*>(interact_mfma_kernel<1>),
                                                              hipFuncAttributeMaxDynamicSharedMemorySize, 136 * 1024);
        if (per_sample > budget && big_lds != hipSuccess) return REC_ERR_DEVICE;
        hipLaunchKernelGGL(interact_mfma_kernel<1>, dim3((unsigned)B), dim3(IT_THREADS), per_sample, s, vecs, B, V, D, out,
                           ldo, zero_to);
    }
    REC_CHECK_LAUNCH();
    return REC_OK;
}
