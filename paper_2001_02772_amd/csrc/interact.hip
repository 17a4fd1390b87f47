// Pairwise-dot feature interaction with strict-lower-triangle packing.
//
// Section II-A ("Feature Interaction") of the DeepRecSys paper: the dense-stack
// output and the pooled embeddings are combined before the predictor stack.
// Here the combination is the DLRM one: all pairwise dot products of the V = T+1
// vectors of a sample, the strict lower triangle packed row by row behind a copy
// of the dense vector.  Per sample this is a V x D matrix times its transpose
// with V and D in the tens: far too small for the matrix cores to pay off and
// dominated by moving [B][V][D] in and [B][D+P] out, so it is plain FMAs from LDS.
#include "rec_common.h"

namespace {

constexpr int IT_THREADS = 256;

__global__ __launch_bounds__(IT_THREADS) void interact_kernel(const float* __restrict__ vecs, int32_t V, int32_t D,
                                                              float* __restrict__ out, int64_t ldo) {
    extern __shared__ __attribute__((aligned(16))) float sm[];
    const int ldv = D + 4;                                  // padded row, 16-byte aligned
    const int tid = threadIdx.x;
    const int64_t b = blockIdx.x;
    const float* __restrict__ v = vecs + b * (int64_t)V * D;
    float* __restrict__ o = out + b * ldo;
    const int d4 = D / 4;
    for (int f = tid; f < V * d4; f += IT_THREADS) {
        const int r = f / d4, c = (f % d4) * 4;
        *reinterpret_cast<float4*>(&sm[r * ldv + c]) = *reinterpret_cast<const float4*>(v + r * D + c);
    }
    __syncthreads();
    for (int d = tid; d < D; d += IT_THREADS) o[d] = sm[d];
    const int P = V * (V - 1) / 2;
    for (int p = tid; p < P; p += IT_THREADS) {
        // row i of the strict lower triangle holds pairs i(i-1)/2 .. i(i+1)/2 - 1
        int i = (int)((1.0f + sqrtf(1.0f + 8.0f * (float)p)) * 0.5f);
        while (i * (i - 1) / 2 > p) --i;
        while (i * (i + 1) / 2 <= p) ++i;
        const int j = p - i * (i - 1) / 2;
        const float* __restrict__ vi = &sm[i * ldv];
        const float* __restrict__ vj = &sm[j * ldv];
        float acc = 0.f;
        for (int c = 0; c < D; c += 4) {
            const float4 a = *reinterpret_cast<const float4*>(vi + c);
            const float4 q = *reinterpret_cast<const float4*>(vj + c);
            acc = fmaf(a.x, q.x, acc);
            acc = fmaf(a.y, q.y, acc);
            acc = fmaf(a.z, q.z, acc);
            acc = fmaf(a.w, q.w, acc);
        }
        o[D + p] = acc;
    }
}

}  // namespace

extern "C" rec_status rec_interact(const float* vecs, int32_t B, int32_t V, int32_t D, float* out, int64_t ldo,
                                   void* stream) {
    if (B < 0 || V < 1) return REC_ERR_BAD_SHAPE;
    if (V > 128 || D < 4 || D > 256 || D % 4) return REC_ERR_UNSUPPORTED;
    if (ldo < (int64_t)D + (int64_t)V * (V - 1) / 2) return REC_ERR_BAD_SHAPE;
    if (B == 0) return REC_OK;
    if (!vecs || !out) return REC_ERR_NULL;
    if (!rec_aligned(vecs, 16)) return REC_ERR_BAD_SHAPE;
    const size_t lds = (size_t)V * (D + 4) * sizeof(float);
    if (lds > 64 * 1024) return REC_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(interact_kernel, dim3((unsigned)B), dim3(IT_THREADS), lds, static_cast<hipStream_t>(stream), vecs,
                       V, D, out, ldo);
    REC_CHECK_LAUNCH();
    return REC_OK;
}
