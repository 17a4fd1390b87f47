// Whole-model forward (Figure 2 of the DeepRecSys paper): embedding bags and the
// dense stack feed the interaction, the predictor stack ends in a sigmoid.
// Also the host-side query splitter of Section IV-A and the status names.
#include <algorithm>
#include <new>
#include <vector>

#include "rec_common.h"
#include "scan_body.h"

struct rec_model {
    int32_t T, D;
    const float* const* tables;
    std::vector<int64_t> rows;
    std::vector<int32_t> bottom_widths, top_widths;
    std::vector<const void*> bottom_W, top_W;
    std::vector<const float*> bottom_b, top_b;
    rec_dtype dt;
    bool concat;             // predictor input = [bottom output | pooled embeddings]
    // The dot interaction's width D + T(T+1)/2 is rarely a multiple of the 16 bytes the FC kernels
    // load at a time (87 for 10 tables of width 32), which would put the first predictor layer on
    // element-wise loads.  The model then owns a copy of that layer's weights with every row
    // zero-padded to `top_k0` columns, and the interaction writes zeros into the matching columns.
    void* top_W0_padded = nullptr;
    bool owns_padded = false;              // allocated by rec_model_create (else the caller's buffer)
    bool prepared = true;                  // the padded copy holds the weights (false until rec_model_prepare)
    const void* top_W0_src = nullptr;      // the caller's unpadded weights of that layer
    std::vector<int32_t> top_widths_run;   // top_widths with [0] = top_k0
    int32_t top_k0;
    int64_t ld_inter;        // row stride of the interaction output (dot) or of the joined row (concat)
};

namespace {

struct ModelWorkspace {
    void* sls;
    size_t sls_bytes;
    float* vecs;
    float* inter;
    void* mlp;
    size_t mlp_bytes;
    size_t total;
};

ModelWorkspace carve(const rec_model* m, int32_t B, void* base) {
    ModelWorkspace w;
    char* p = static_cast<char*>(base);
    const int32_t V = m->T + 1;
    w.sls = p;
    w.sls_bytes = rec_sls_workspace_bytes(m->T, B);
    p += w.sls_bytes;
    w.vecs = reinterpret_cast<float*>(p);
    if (!m->concat) p += rec_round_up((size_t)B * V * m->D * sizeof(float), 256);
    w.inter = reinterpret_cast<float*>(p);
    p += rec_round_up((size_t)B * m->ld_inter * sizeof(float), 256);
    w.mlp = p;
    const size_t a = m->bottom_W.empty() ? 0 : rec_mlp_workspace_bytes(m->bottom_widths.data(), (int32_t)m->bottom_W.size(), B, m->dt);
    const size_t c = rec_mlp_workspace_bytes(m->top_widths_run.data(), (int32_t)m->top_W.size(), B, m->dt);
    w.mlp_bytes = a > c ? a : c;
    p += w.mlp_bytes;
    w.total = (size_t)(p - static_cast<char*>(base));
    return w;
}

// dst[b][0..F) = src[b][0..F): dense features that skip the dense stack (Section II-A, Wide&Deep).
// The first `scan_tiles` blocks of the launch do the bag-offsets scan instead (see scan_body.h), so
// a model without a dense stack does not pay a launch for either.
__global__ __launch_bounds__(SCAN_THREADS) void copy_rows_scan_kernel(const float* __restrict__ src, float* __restrict__ dst,
                                                                      int32_t B, int32_t F, int64_t ld_dst,
                                                                      const int32_t* __restrict__ len, int64_t n_bags,
                                                                      int64_t* __restrict__ off, int vec_ok, int scan_tiles) {
    if ((int)blockIdx.x < scan_tiles) {
        offsets_block(len, n_bags, off, vec_ok, (int)blockIdx.x, true);
        return;
    }
    const int64_t n4 = (int64_t)B * (F / 4);
    const int64_t first = (int64_t)(blockIdx.x - scan_tiles) * SCAN_THREADS + threadIdx.x;
    const int64_t step = (int64_t)(gridDim.x - scan_tiles) * SCAN_THREADS;
    for (int64_t i = first; i < n4; i += step) {
        const int64_t b = i / (F / 4);
        const int32_t c = (int32_t)(i - b * (F / 4)) * 4;
        *reinterpret_cast<float4*>(dst + b * ld_dst + c) = *reinterpret_cast<const float4*>(src + b * F + c);
    }
}

// dst[r][0..kp) = src[r][0..k) followed by zeros, rows of `elt`-byte elements.
__global__ __launch_bounds__(256) void pad_rows_kernel(const unsigned char* __restrict__ src, unsigned char* __restrict__ dst,
                                                       int64_t rows, int32_t k, int32_t kp, int32_t elt) {
    const int64_t n = rows * kp;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = i / kp;
        const int32_t c = (int32_t)(i - r * kp);
        for (int32_t b = 0; b < elt; ++b) dst[i * elt + b] = c < k ? src[(r * k + c) * elt + b] : (unsigned char)0;
    }
}

// Columns the first predictor layer's k is padded to (k itself when no padding is needed).
int32_t padded_k0(int32_t k0, rec_dtype dt, bool concat) {
    int32_t align = (dt == REC_BF16) ? 8 : 4;                       // elements per 16-byte load
    // a wide first predictor layer runs on the tiled matrix kernels when its k is a multiple of their
    // 128-byte slice (884 -> 896 for 40 tables of width 64)
    if (k0 >= 256) align *= 8;
    return (!concat && k0 % align != 0) ? (k0 + align - 1) / align * align : k0;
}

}  // namespace

extern "C" {

const char* rec_status_string(rec_status s) {
    switch (s) {
        case REC_OK: return "REC_OK";
        case REC_ERR_NULL: return "REC_ERR_NULL";
        case REC_ERR_BAD_SHAPE: return "REC_ERR_BAD_SHAPE";
        case REC_ERR_NEGATIVE_LENGTH: return "REC_ERR_NEGATIVE_LENGTH";
        case REC_ERR_LENGTHS_MISMATCH: return "REC_ERR_LENGTHS_MISMATCH";
        case REC_ERR_INDEX_RANGE: return "REC_ERR_INDEX_RANGE";
        case REC_ERR_WORKSPACE: return "REC_ERR_WORKSPACE";
        case REC_ERR_UNSUPPORTED: return "REC_ERR_UNSUPPORTED";
        case REC_ERR_DEVICE: return "REC_ERR_DEVICE";
    }
    return "REC_ERR_UNKNOWN";
}

int64_t rec_split_query(int64_t n, int64_t batch, int64_t* start, int64_t* count) {
    if (n < 0 || batch < 1) return -1;
    const int64_t full = n / batch, rem = n % batch;
    for (int64_t k = 0; k < full; ++k) {
        if (start) start[k] = k * batch;
        if (count) count[k] = batch;
    }
    if (rem) {
        if (start) start[full] = full * batch;
        if (count) count[full] = rem;
    }
    return full + (rem ? 1 : 0);
}

rec_status rec_model_create(const rec_model_desc* d, rec_model** out) {
    if (!d || !out) return REC_ERR_NULL;
    *out = nullptr;
    if (!d->tables || !d->rows || !d->bottom_widths || !d->top_widths || !d->top_W || !d->top_b) return REC_ERR_NULL;
    if (d->n_bottom > 0 && (!d->bottom_W || !d->bottom_b)) return REC_ERR_NULL;
    if (d->interaction != REC_INTERACT_DOT && d->interaction != REC_INTERACT_CONCAT) return REC_ERR_UNSUPPORTED;
    const bool concat = d->interaction == REC_INTERACT_CONCAT;
    if (d->T < 1 || d->n_bottom < (concat ? 0 : 1) || d->n_top < 1) return REC_ERR_BAD_SHAPE;
    if (d->T > 127 || d->D < 4 || d->D > 256 || d->D % 4) return REC_ERR_UNSUPPORTED;
    if (d->mlp_dtype != REC_F32 && d->mlp_dtype != REC_BF16) return REC_ERR_UNSUPPORTED;
    for (int32_t l = 0; l <= d->n_bottom; ++l)
        if (d->bottom_widths[l] < 1) return REC_ERR_BAD_SHAPE;
    for (int32_t l = 0; l <= d->n_top; ++l)
        if (d->top_widths[l] < 1) return REC_ERR_BAD_SHAPE;
    const int32_t V = d->T + 1;
    const int32_t X = d->bottom_widths[d->n_bottom];
    if (concat) {
        if ((int64_t)d->top_widths[0] != (int64_t)X + (int64_t)d->T * d->D || d->top_widths[d->n_top] != 1) return REC_ERR_BAD_SHAPE;
        if (X % 4) return REC_ERR_UNSUPPORTED;
    } else {
        if (X != d->D) return REC_ERR_BAD_SHAPE;
        if (d->top_widths[0] != d->D + V * (V - 1) / 2 || d->top_widths[d->n_top] != 1) return REC_ERR_BAD_SHAPE;
    }
    for (int32_t t = 0; t < d->T; ++t) {
        if (d->rows[t] < 1) return REC_ERR_BAD_SHAPE;
        if (d->rows[t] > 2147483647LL) return REC_ERR_UNSUPPORTED;
    }
    for (int32_t l = 0; l < d->n_bottom; ++l)
        if (!d->bottom_W[l] || !d->bottom_b[l]) return REC_ERR_NULL;
    for (int32_t l = 0; l < d->n_top; ++l)
        if (!d->top_W[l] || !d->top_b[l]) return REC_ERR_NULL;
    rec_model* m = new (std::nothrow) rec_model;
    if (!m) return REC_ERR_DEVICE;
    m->T = d->T;
    m->D = d->D;
    m->tables = d->tables;
    m->rows.assign(d->rows, d->rows + d->T);
    m->bottom_widths.assign(d->bottom_widths, d->bottom_widths + d->n_bottom + 1);
    m->top_widths.assign(d->top_widths, d->top_widths + d->n_top + 1);
    if (d->n_bottom > 0) {
        m->bottom_W.assign(d->bottom_W, d->bottom_W + d->n_bottom);
        m->bottom_b.assign(d->bottom_b, d->bottom_b + d->n_bottom);
    }
    m->top_W.assign(d->top_W, d->top_W + d->n_top);
    m->top_b.assign(d->top_b, d->top_b + d->n_top);
    m->dt = d->mlp_dtype;
    m->concat = concat;
    m->top_widths_run = m->top_widths;
    const int32_t k0 = d->top_widths[0];
    const int32_t kp = padded_k0(k0, d->mlp_dtype, concat);
    m->top_k0 = kp;
    if (kp != k0) {
        const size_t need = rec_model_padded_weight_bytes(d);
        m->top_W0_src = d->top_W[0];
        m->top_widths_run[0] = kp;
        if (d->padded_weights) {
            // the caller's buffer: nothing touches the device here; rec_model_prepare fills it
            if (d->padded_weights_bytes < need || !rec_aligned(d->padded_weights, 256)) {
                delete m;
                return REC_ERR_WORKSPACE;
            }
            m->top_W0_padded = d->padded_weights;
            m->prepared = false;
        } else {
            const size_t elt = (d->mlp_dtype == REC_BF16) ? 2 : 4;
            const size_t n_out = (size_t)d->top_widths[1];
            void* padded = nullptr;
            if (hipMalloc(&padded, need) != hipSuccess) {
                delete m;
                return REC_ERR_DEVICE;
            }
            if (hipMemset(padded, 0, need) != hipSuccess ||
                hipMemcpy2D(padded, kp * elt, d->top_W[0], k0 * elt, k0 * elt, n_out, hipMemcpyDeviceToDevice) != hipSuccess ||
                hipDeviceSynchronize() != hipSuccess) {
                (void)hipFree(padded);
                delete m;
                return REC_ERR_DEVICE;
            }
            m->top_W0_padded = padded;
            m->owns_padded = true;
        }
        m->top_W[0] = m->top_W0_padded;
    }
    m->ld_inter = (m->top_k0 + 3) / 4 * 4;
    *out = m;
    return REC_OK;
}

size_t rec_model_padded_weight_bytes(const rec_model_desc* d) {
    if (!d || !d->top_widths || d->n_top < 1) return 0;
    if (d->mlp_dtype != REC_F32 && d->mlp_dtype != REC_BF16) return 0;
    const int32_t k0 = d->top_widths[0];
    if (k0 < 1 || d->top_widths[1] < 1) return 0;
    const int32_t kp = padded_k0(k0, d->mlp_dtype, d->interaction == REC_INTERACT_CONCAT);
    if (kp == k0) return 0;
    return rec_round_up((size_t)d->top_widths[1] * kp * (d->mlp_dtype == REC_BF16 ? 2 : 4), 256);
}

rec_status rec_model_prepare(rec_model* m, void* stream) {
    if (!m) return REC_ERR_NULL;
    if (m->prepared) return REC_OK;
    const int32_t k0 = m->top_widths[0], kp = m->top_k0, elt = (m->dt == REC_BF16) ? 2 : 4;
    const int64_t rows = m->top_widths[1];
    const int64_t n = rows * kp;
    hipLaunchKernelGGL(pad_rows_kernel, dim3((unsigned)std::min<int64_t>((n + 255) / 256, 1024)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<const unsigned char*>(m->top_W0_src),
                       static_cast<unsigned char*>(m->top_W0_padded), rows, k0, kp, elt);
    REC_CHECK_LAUNCH();
    m->prepared = true;
    return REC_OK;
}

void rec_model_destroy(rec_model* m) {
    if (!m) return;
    if (m->top_W0_padded && m->owns_padded) (void)hipFree(m->top_W0_padded);
    delete m;
}

size_t rec_model_workspace_bytes(const rec_model* m, int32_t B_max) {
    if (!m || B_max < 0) return 0;
    return carve(m, B_max, nullptr).total;
}

rec_status rec_model_forward(const rec_model* m, const float* dense, const int32_t* indices, int64_t n_indices,
                             const int32_t* lengths, int32_t B, float* prob, void* workspace,
                             size_t workspace_bytes, void* stream) {
    if (!m) return REC_ERR_NULL;
    if (B < 0 || n_indices < 0) return REC_ERR_BAD_SHAPE;
    if (!m->prepared) return REC_ERR_BAD_SHAPE;                     // rec_model_prepare has not run
    if (B == 0) return REC_OK;
    if (!dense || !lengths || !prob || (n_indices > 0 && !indices)) return REC_ERR_NULL;
    if (!workspace || !rec_aligned(workspace, 256)) return REC_ERR_WORKSPACE;
    const ModelWorkspace w = carve(m, B, workspace);
    if (workspace_bytes < w.total) return REC_ERR_WORKSPACE;
    const int32_t V = m->T + 1, D = m->D;
    const rec_scan_job scan = {lengths, (int64_t)m->T * B, rec_sls_workspace_offsets(w.sls)};

    if (m->concat) {
        // [ x | E_0 .. E_{T-1} ] is assembled in place: the pooling kernel and the dense stack (or
        // the copy of the dense features) write their columns of the joined rows directly
        const int32_t X = m->bottom_widths.back();
        const int64_t ldc = m->ld_inter;
        if (m->bottom_W.empty()) {
            if (!rec_aligned(dense, 16)) return REC_ERR_BAD_SHAPE;  // the row copy below loads 16 bytes at a time
            rec_status st = rec_sls_forward_step(m->tables, m->rows.data(), m->T, D, indices, n_indices, lengths, B,
                                                 w.inter + X, ldc, D, w.sls, w.sls_bytes, stream, REC_SLS_CHECK_ONLY);
            if (st != REC_OK) return st;
            int tiles = rec_scan_parallel_tiles(scan.n);
            if (tiles < 1) {                                         // very long batch: the scan walks its tiles in one block
                st = rec_scan_launch(scan, static_cast<hipStream_t>(stream));
                if (st != REC_OK) return st;
                tiles = 0;
            }
            const int64_t n4 = (int64_t)B * (X / 4);
            const unsigned blocks = (unsigned)std::min<int64_t>((n4 + SCAN_THREADS - 1) / SCAN_THREADS, 1024);
            hipLaunchKernelGGL(copy_rows_scan_kernel, dim3(blocks + tiles), dim3(SCAN_THREADS), 0,
                               static_cast<hipStream_t>(stream), dense, w.inter, B, X, ldc, scan.lengths, scan.n, scan.offsets,
                               (int)rec_aligned(scan.lengths, 16), tiles);
            REC_CHECK_LAUNCH();
            st = rec_sls_forward_step(m->tables, m->rows.data(), m->T, D, indices, n_indices, lengths, B, w.inter + X, ldc,
                                      D, w.sls, w.sls_bytes, stream, REC_SLS_POOL_ONLY);
            if (st != REC_OK) return st;
        } else {
            // the offsets scan rides with the dense stack's first launch; the pooling follows both
            rec_status st = rec_sls_forward_step(m->tables, m->rows.data(), m->T, D, indices, n_indices, lengths, B,
                                                 w.inter + X, ldc, D, w.sls, w.sls_bytes, stream, REC_SLS_CHECK_ONLY);
            if (st != REC_OK) return st;
            st = rec_mlp_forward_scan(m->bottom_W.data(), m->bottom_b.data(), m->bottom_widths.data(),
                                      (int32_t)m->bottom_W.size(), m->dt, REC_ACT_RELU, REC_ACT_RELU, dense,
                                      m->bottom_widths[0], w.inter, ldc, B, w.mlp, w.mlp_bytes, stream, &scan);
            if (st != REC_OK) return st;
            st = rec_sls_forward_step(m->tables, m->rows.data(), m->T, D, indices, n_indices, lengths, B, w.inter + X, ldc,
                                      D, w.sls, w.sls_bytes, stream, REC_SLS_POOL_ONLY);
            if (st != REC_OK) return st;
        }
        return rec_mlp_forward(m->top_W.data(), m->top_b.data(), m->top_widths.data(), (int32_t)m->top_W.size(), m->dt,
                               REC_ACT_RELU, REC_ACT_SIGMOID, w.inter, ldc, prob, 1, B, w.mlp, w.mlp_bytes, stream);
    }

    // dense stack first: the offsets scan rides with its first launch, the pooling follows both
    rec_status st = rec_sls_forward_step(m->tables, m->rows.data(), m->T, D, indices, n_indices, lengths, B, w.vecs + D,
                                         (int64_t)V * D, D, w.sls, w.sls_bytes, stream, REC_SLS_CHECK_ONLY);
    if (st != REC_OK) return st;
    st = rec_mlp_forward_scan(m->bottom_W.data(), m->bottom_b.data(), m->bottom_widths.data(),
                              (int32_t)m->bottom_W.size(), m->dt, REC_ACT_RELU, REC_ACT_RELU, dense, m->bottom_widths[0],
                              w.vecs, (int64_t)V * D, B, w.mlp, w.mlp_bytes, stream, &scan);
    if (st != REC_OK) return st;
    st = rec_sls_forward_step(m->tables, m->rows.data(), m->T, D, indices, n_indices, lengths, B, w.vecs + D,
                              (int64_t)V * D, D, w.sls, w.sls_bytes, stream, REC_SLS_POOL_ONLY);
    if (st != REC_OK) return st;
    // the interaction runs inside the predictor stack's first launch when it can, else on its own
    const rec_interact_job inter = {w.vecs, V, D, w.inter, m->ld_inter, m->top_k0};
    return rec_mlp_forward_scan(m->top_W.data(), m->top_b.data(), m->top_widths_run.data(), (int32_t)m->top_W.size(), m->dt,
                                REC_ACT_RELU, REC_ACT_SIGMOID, w.inter, m->ld_inter, prob, 1, B, w.mlp, w.mlp_bytes, stream,
                                nullptr, &inter);
}

}  // extern "C"
