/* CPU oracle for batched DLRM-style inference.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, by-the-definition implementation of what the GPU library
 * computes, written from the model description in Section II-A of the
 * DeepRecSys paper ("Key Components in Neural Recommendation Models") and the
 * shape table (Table I).  It shares no code with the GPU path.  Only tests, the
 * smoke check and the benchmark's CPU-baseline leg may call it; the product
 * never does.
 *
 * All floating-point sums are accumulated in fp64 and rounded once to fp32,
 * unless a function says otherwise.  Loops run in the order the definition
 * states; there is no blocking, vectorisation or fusion.  The only concession
 * to run time is an OpenMP "parallel for" over independent samples or bags
 * (the request-level parallelism of Section IV-A), which does not change any
 * result.
 *
 * Every function here is pinned by tests that do not use the function itself:
 * hand-computed bags, closed forms, invariants and NumPy / PyTorch-CPU library
 * routines.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_OK = 0, ORC_ERR_NULL = 1, ORC_ERR_BAD_SHAPE = 2, ORC_ERR_NEGATIVE_LENGTH = 3,
       ORC_ERR_LENGTHS_MISMATCH = 4, ORC_ERR_INDEX_RANGE = 5 };
enum { ORC_ACT_NONE = 0, ORC_ACT_RELU = 1, ORC_ACT_SIGMOID = 2 };

static int g_threads = 1;

void orc_set_threads(int n) { g_threads = n < 1 ? 1 : n; }

int orc_get_threads(void) {
#ifdef _OPENMP
    return g_threads;
#else
    return 1;
#endif
}

/* Round an fp32 value to the nearest bf16 (ties to even), returned as fp32.
 * bf16 keeps the top 16 bits of the fp32 pattern.  NaN stays NaN. */
float orc_bf16_round(float x) {
    uint32_t u;
    memcpy(&u, &x, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) {
        u |= 0x00400000u;           /* quiet the NaN, keep it a NaN */
        u &= 0xffff0000u;
    } else {
        uint32_t lsb = (u >> 16) & 1u;
        u += 0x7fffu + lsb;
        u &= 0xffff0000u;
    }
    memcpy(&x, &u, 4);
    return x;
}

void orc_bf16_round_array(const float* x, float* y, int64_t n) {
    for (int64_t i = 0; i < n; ++i) y[i] = orc_bf16_round(x[i]);
}

/* Input check for the sparse side (Section II-A, "Embedding Table Access": the
 * sparse inputs index into specific rows of their table).  Bags are table-major:
 * bag t*B+b holds the lookups of sample b into table t.
 *   - every length >= 0                       else ORC_ERR_NEGATIVE_LENGTH
 *   - sum of lengths (64-bit) == n_indices    else ORC_ERR_LENGTHS_MISMATCH
 *   - every index of table t in [0, rows[t])  else ORC_ERR_INDEX_RANGE
 * n_bad = number of out-of-range indices, first_bad = flat position of the
 * first one (-1 if none); both are only meaningful when the first two checks
 * pass. */
int orc_validate(const int64_t* rows, int32_t T, const int32_t* indices, int64_t n_indices,
                 const int32_t* lengths, int32_t B, int64_t* n_bad, int64_t* first_bad) {
    *n_bad = 0;
    *first_bad = -1;
    int64_t total = 0;
    for (int64_t i = 0; i < (int64_t)T * B; ++i) {
        if (lengths[i] < 0) return ORC_ERR_NEGATIVE_LENGTH;
        total += lengths[i];
    }
    if (total != n_indices) return ORC_ERR_LENGTHS_MISMATCH;
    int64_t pos = 0;
    for (int32_t t = 0; t < T; ++t)
        for (int32_t b = 0; b < B; ++b)
            for (int32_t k = 0; k < lengths[(int64_t)t * B + b]; ++k, ++pos)
                if (indices[pos] < 0 || (int64_t)indices[pos] >= rows[t]) {
                    if (*n_bad == 0) *first_bad = pos;
                    ++*n_bad;
                }
    return *n_bad ? ORC_ERR_INDEX_RANGE : ORC_OK;
}

/* Exclusive prefix sum of the bag lengths: off[0] = 0, off[i+1] = off[i] + lengths[i]. */
void orc_offsets(const int32_t* lengths, int64_t n_bags, int64_t* off) {
    off[0] = 0;
    for (int64_t i = 0; i < n_bags; ++i) off[i + 1] = off[i] + lengths[i];
}

/* Embedding lookup with sum pooling (Section II-A, "Embedding Table Access";
 * Table I, pooling = Sum): for bag (t, b)
 *     E[b][t][:] = sum over k < L  of  Table_t[ idx[off + k] ][:]
 * unweighted, duplicates counted as often as they occur, empty bag -> zeros.
 * Element (b, t, d) is written to out[b*stride_b + t*stride_t + d].
 *   out       fp64-accumulated sum rounded once to fp32 (the reference value)
 *   out_seq   optional: plain fp32 running sum in lookup order
 *   out_abs   optional: fp64 sum of |x|, same addressing as out, for error bounds */
void orc_sls(const float* const* tables, int32_t T, int32_t D, const int32_t* indices,
             const int64_t* off, int32_t B, float* out, int64_t stride_b, int64_t stride_t,
             float* out_seq, double* out_abs) {
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int32_t b = 0; b < B; ++b) {
        double* acc = (double*)malloc(sizeof(double) * D * 2);
        float* seq = (float*)malloc(sizeof(float) * D);
        double* aabs = acc + D;
        for (int32_t t = 0; t < T; ++t) {
            const int64_t bag = (int64_t)t * B + b;
            for (int32_t d = 0; d < D; ++d) { acc[d] = 0.0; aabs[d] = 0.0; seq[d] = 0.0f; }
            for (int64_t p = off[bag]; p < off[bag + 1]; ++p) {
                const float* row = tables[t] + (int64_t)indices[p] * D;
                for (int32_t d = 0; d < D; ++d) {
                    acc[d] += (double)row[d];
                    aabs[d] += fabs((double)row[d]);
                    seq[d] = seq[d] + row[d];
                }
            }
            const int64_t o = b * stride_b + t * stride_t;
            for (int32_t d = 0; d < D; ++d) {
                out[o + d] = (float)acc[d];
                if (out_seq) out_seq[o + d] = seq[d];
                if (out_abs) out_abs[o + d] = aabs[d];
            }
        }
        free(acc);
        free(seq);
    }
}

static float apply_act(double z, int act) {
    if (act == ORC_ACT_RELU) return (float)(z > 0.0 ? z : 0.0);
    if (act == ORC_ACT_SIGMOID) return (float)(1.0 / (1.0 + exp(-z)));
    return (float)z;
}

/* One fully-connected layer (Section II-A, "Features": dense inputs go through a
 * stack of fully-connected layers; "Product Ranking": the predictor stack ends
 * in a click probability):
 *     y[b][o] = act( bias[o] + sum_i x[b][i] * W[o][i] )
 * W is [n_out][n_in] row-major.  With bf16_operands != 0, x and W are first
 * rounded to bf16 (ties to even).  Products, the sum, the bias add and the
 * activation are all evaluated in fp64; the result is rounded once to fp32. */
void orc_fc(const float* x, int64_t ldx, const float* W, const float* bias, int32_t B,
            int32_t n_in, int32_t n_out, int32_t act, int32_t bf16_operands, float* y, int64_t ldy) {
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int32_t b = 0; b < B; ++b) {
        for (int32_t o = 0; o < n_out; ++o) {
            double acc = 0.0;
            for (int32_t i = 0; i < n_in; ++i) {
                float xv = x[b * ldx + i], wv = W[(int64_t)o * n_in + i];
                if (bf16_operands) { xv = orc_bf16_round(xv); wv = orc_bf16_round(wv); }
                acc += (double)xv * (double)wv;
            }
            y[b * ldy + o] = apply_act(acc + (double)bias[o], act);
        }
    }
}

/* A stack of FC layers: hidden layers use hidden_act, the last uses final_act.
 * W[l] is [widths[l+1]][widths[l]].  Activations between layers are fp32. */
void orc_mlp(const float* const* W, const float* const* bias, const int32_t* widths,
             int32_t n_layers, int32_t bf16_operands, int32_t hidden_act, int32_t final_act,
             const float* x, int64_t ldx, float* y, int64_t ldy, int32_t B) {
    const float* cur = x;
    int64_t ld = ldx;
    float* tmp = NULL;
    for (int32_t l = 0; l < n_layers; ++l) {
        const int last = (l == n_layers - 1);
        float* dst = last ? y : (float*)malloc(sizeof(float) * (size_t)B * widths[l + 1]);
        const int64_t ldd = last ? ldy : widths[l + 1];
        orc_fc(cur, ld, W[l], bias[l], B, widths[l], widths[l + 1], last ? final_act : hidden_act,
               bf16_operands, dst, ldd);
        free(tmp);
        tmp = last ? NULL : dst;
        cur = dst;
        ld = ldd;
    }
}

/* Pairwise-dot feature interaction (Section II-A, "Feature Interaction": the
 * dense-stack output and the pooled embeddings are combined before the
 * predictor stack).  vecs is [B][V][D]; slot 0 is the dense-stack output,
 * slots 1..V-1 the pooled embeddings.  For each sample
 *     out[b] = [ vecs[b][0][0..D) ,  <vecs[b][i], vecs[b][j]>  for i = 1..V-1, j = 0..i-1 ]
 * i.e. the D values of slot 0 copied unchanged, then the strict lower triangle
 * of V V^T in row-major order.  Width D + V(V-1)/2, row stride ldo. */
void orc_interact(const float* vecs, int32_t B, int32_t V, int32_t D, float* out, int64_t ldo) {
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int32_t b = 0; b < B; ++b) {
        const float* v = vecs + (int64_t)b * V * D;
        float* o = out + b * ldo;
        for (int32_t d = 0; d < D; ++d) o[d] = v[d];
        int64_t p = D;
        for (int32_t i = 1; i < V; ++i)
            for (int32_t j = 0; j < i; ++j) {
                double acc = 0.0;
                for (int32_t d = 0; d < D; ++d) acc += (double)v[i * D + d] * (double)v[j * D + d];
                o[p++] = (float)acc;
            }
    }
}

/* Whole model (Figure 2): offsets -> SLS into slots 1..T of [B][T+1][D];
 * bottom stack (ReLU on every layer) into slot 0; interaction; top stack (ReLU
 * on hidden layers, sigmoid on the 1-wide last layer) -> prob[B].
 * Returns ORC_OK or the validator's status; nothing is computed on bad input. */
int orc_model_forward(const float* const* tables, const int64_t* rows, int32_t T, int32_t D,
                      const float* const* Wb, const float* const* bb, const int32_t* wb, int32_t nb,
                      const float* const* Wt, const float* const* bt, const int32_t* wt, int32_t nt,
                      int32_t bf16_operands, const float* dense, const int32_t* indices,
                      int64_t n_indices, const int32_t* lengths, int32_t B, float* prob) {
    if (wb[nb] != D || wt[0] != D + (T + 1) * T / 2 || wt[nt] != 1) return ORC_ERR_BAD_SHAPE;
    int64_t n_bad, first_bad;
    int st = orc_validate(rows, T, indices, n_indices, lengths, B, &n_bad, &first_bad);
    if (st != ORC_OK) return st;
    if (B == 0) return ORC_OK;
    const int32_t V = T + 1;
    int64_t* off = (int64_t*)malloc(sizeof(int64_t) * ((size_t)T * B + 1));
    float* vecs = (float*)malloc(sizeof(float) * (size_t)B * V * D);
    float* inter = (float*)malloc(sizeof(float) * (size_t)B * wt[0]);
    orc_offsets(lengths, (int64_t)T * B, off);
    orc_sls(tables, T, D, indices, off, B, vecs + D, (int64_t)V * D, D, NULL, NULL);
    orc_mlp(Wb, bb, wb, nb, bf16_operands, ORC_ACT_RELU, ORC_ACT_RELU, dense, wb[0], vecs,
            (int64_t)V * D, B);
    orc_interact(vecs, B, V, D, inter, wt[0]);
    orc_mlp(Wt, bt, wt, nt, bf16_operands, ORC_ACT_RELU, ORC_ACT_SIGMOID, inter, wt[0], prob, 1, B);
    free(off);
    free(vecs);
    free(inter);
    return ORC_OK;
}

/* Concatenating models (Table I: NCF, Wide&Deep use "Concat" where DLRM interacts; Section II-A:
 * dense features that bypass the Dense-FC stack are joined directly with the embedding outputs).
 * Predictor input of sample b = [ x_b | E[b][0][:] | ... | E[b][T-1][:] ], where x_b is the output
 * of the dense stack (ReLU on every layer), or the dense features themselves when that stack has
 * no layers (nb == 0, wb[0] = number of dense features), and E is the pooled embedding of each
 * table (one lookup per bag in the paper's concat models; any bag length is summed).  Top stack
 * as in orc_model_forward.  wt[0] must equal wb[nb] + T*D. */
int orc_model_forward_concat(const float* const* tables, const int64_t* rows, int32_t T, int32_t D,
                             const float* const* Wb, const float* const* bb, const int32_t* wb, int32_t nb,
                             const float* const* Wt, const float* const* bt, const int32_t* wt, int32_t nt,
                             int32_t bf16_operands, const float* dense, const int32_t* indices,
                             int64_t n_indices, const int32_t* lengths, int32_t B, float* prob) {
    const int32_t X = wb[nb];
    if (wt[0] != X + T * D || wt[nt] != 1) return ORC_ERR_BAD_SHAPE;
    int64_t n_bad, first_bad;
    int st = orc_validate(rows, T, indices, n_indices, lengths, B, &n_bad, &first_bad);
    if (st != ORC_OK) return st;
    if (B == 0) return ORC_OK;
    const int64_t Wc = wt[0];
    int64_t* off = (int64_t*)malloc(sizeof(int64_t) * ((size_t)T * B + 1));
    float* cat = (float*)malloc(sizeof(float) * (size_t)B * Wc);
    orc_offsets(lengths, (int64_t)T * B, off);
    orc_sls(tables, T, D, indices, off, B, cat + X, Wc, D, NULL, NULL);
    if (nb > 0) {
        orc_mlp(Wb, bb, wb, nb, bf16_operands, ORC_ACT_RELU, ORC_ACT_RELU, dense, wb[0], cat, Wc, B);
    } else {
        for (int32_t b = 0; b < B; ++b)
            for (int32_t f = 0; f < X; ++f) cat[b * Wc + f] = dense[(int64_t)b * X + f];
    }
    orc_mlp(Wt, bt, wt, nt, bf16_operands, ORC_ACT_RELU, ORC_ACT_SIGMOID, cat, Wc, prob, 1, B);
    free(off);
    free(cat);
    return ORC_OK;
}

/* Split a query of n items into consecutive sub-batches of size Bsz (Section
 * IV-A: a query is divided into requests of a given batch size): floor(n/Bsz)
 * full ones, then one of n mod Bsz if that is non-zero.  Writes (start, count)
 * pairs and returns how many; pass NULL pointers to only count. */
int64_t orc_split_query(int64_t n, int64_t Bsz, int64_t* start, int64_t* count) {
    int64_t k = 0;
    for (int64_t s = 0; s < n; s += Bsz, ++k) {
        if (start) start[k] = s;
        if (count) count[k] = (n - s < Bsz) ? n - s : Bsz;
    }
    return k;
}

/* ------------------------------------------------------------------------
 * Query serving and the batch-size hill climb (Sections III-C, IV-A, IV-C).
 * ---------------------------------------------------------------------- */

/* Time to serve a query of n items cut into requests of size B (Section IV-A): floor(n/B)
 * requests of B items and one of n mod B items, run one after another on one device.
 * t[b] = seconds for one request of b items, b = 1..B (t[0] unused). */
double orc_query_service(int64_t n, int64_t B, const double* t) {
    double s = 0.0;
    for (int64_t k = 0; k < n / B; ++k) s += t[B];
    if (n % B) s += t[n % B];
    return s;
}

/* Queries served first-come-first-served by one device: a query starts when it has arrived
 * and the previous one has finished; its latency is finish - arrival (queueing included). */
void orc_fifo_latencies(const double* arrival, const double* service, int64_t n, double* latency) {
    double prev_finish = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        const double start = (i > 0 && prev_finish > arrival[i]) ? prev_finish : arrival[i];
        prev_finish = start + service[i];
        latency[i] = prev_finish - arrival[i];
    }
}

static int cmp_double(const void* a, const void* b) {
    const double x = *(const double*)a, y = *(const double*)b;
    return (x > y) - (x < y);
}

/* Nearest-rank percentile: the smallest sample v such that at least a fraction p of the
 * samples is <= v, i.e. sorted[ceil(p*n) - 1].  p in (0, 1]. */
double orc_percentile(const double* x, int64_t n, double p) {
    double* s = (double*)malloc(sizeof(double) * (size_t)n);
    memcpy(s, x, sizeof(double) * (size_t)n);
    qsort(s, (size_t)n, sizeof(double), cmp_double);
    int64_t k = (int64_t)ceil(p * (double)n) - 1;
    if (k < 0) k = 0;
    if (k > n - 1) k = n - 1;
    const double v = s[k];
    free(s);
    return v;
}

static int orc_rate_ok(const double* unit_arrival, const double* service, int64_t n, double p, double sla,
                       double rate, double* arr, double* lat) {
    for (int64_t i = 0; i < n; ++i) arr[i] = unit_arrival[i] / rate;
    orc_fifo_latencies(arr, service, n, lat);
    return orc_percentile(lat, n, p) <= sla;
}

/* Latency-bounded throughput (Section III-B: QPS under a p95 tail-latency target): the largest
 * arrival rate (queries/s) at which the p-th percentile latency stays <= sla.  Arrivals are
 * unit_arrival[i] / rate (unit_arrival = arrival times of a rate-1 Poisson process), so a higher
 * rate only compresses the same arrival pattern and latencies grow monotonically with it.
 * 0 if the target is missed even without queueing.  The rate is bracketed by doubling from 1
 * (halving if 1 is already too fast), then bisected `iters` times; the feasible end is returned. */
double orc_max_qps(const double* unit_arrival, const double* service, int64_t n, double p, double sla, int32_t iters) {
    if (n <= 0) return 0.0;
    if (orc_percentile(service, n, p) > sla) return 0.0;
    double* arr = (double*)malloc(sizeof(double) * (size_t)n);
    double* lat = (double*)malloc(sizeof(double) * (size_t)n);
    double lo = 1.0, hi = 1.0;
    if (orc_rate_ok(unit_arrival, service, n, p, sla, 1.0, arr, lat)) {
        hi = 2.0;
        while (hi < 1e15 && orc_rate_ok(unit_arrival, service, n, p, sla, hi, arr, lat)) { lo = hi; hi *= 2.0; }
    } else {
        lo = 0.5;
        while (lo > 1e-15 && !orc_rate_ok(unit_arrival, service, n, p, sla, lo, arr, lat)) { hi = lo; lo *= 0.5; }
    }
    for (int32_t k = 0; k < iters; ++k) {
        const double mid = 0.5 * (lo + hi);
        if (orc_rate_ok(unit_arrival, service, n, p, sla, mid, arr, lat)) lo = mid; else hi = mid;
    }
    free(arr);
    free(lat);
    return lo;
}

/* Batch-size hill climb (Section IV-C): start at the first candidate (unit batch size) and move
 * to the next larger one as long as the sustainable query rate does not drop: stop at the first
 * step that lowers it (a step that leaves it unchanged, such as one between two batch sizes that both miss
 * the latency target, is taken).  qps[i] = achievable QPS with the i-th candidate batch size.
 * Returns the index kept. */
int64_t orc_hill_climb(const double* qps, int64_t n_candidates) {
    int64_t i = 0;
    while (i + 1 < n_candidates && qps[i + 1] >= qps[i]) ++i;
    return i;
}

/* ------------------------------------------------------------------------
 * Two tiers: CPU workers and one accelerator (Section IV-B "Leverage parallelism with
 * specialized hardware", Section IV-C second paragraph).
 * ---------------------------------------------------------------------- */

/* Queries whose size reaches the threshold tau go whole to the accelerator: one device, first
 * come first served, g[m] seconds for a query of m items (transfer included).  The others are
 * cut into requests of batch size B (Section IV-A) that run on k identical CPU workers, one
 * request per worker at a time (the paper runs one request per core): requests are handed out
 * in arrival order, each to the worker that is free first, c[b] seconds for a request of b
 * items; a query is done when its last request is done.  latency = done - arrival.
 * tau = 1 sends every query to the accelerator (the paper's starting point of the climb),
 * tau above the largest size sends none.  free_at: scratch, k doubles. */
static void orc_two_tier_run(const double* arrival, const int64_t* size, int64_t n, int64_t tau, int64_t B,
                             const double* c, int32_t k, const double* g, double* latency, double* free_at) {
    double gpu_free = 0.0;
    for (int32_t w = 0; w < k; ++w) free_at[w] = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        const int64_t m = size[i];
        double done = arrival[i];
        if (m >= tau) {
            const double start = gpu_free > arrival[i] ? gpu_free : arrival[i];
            gpu_free = start + g[m];
            done = gpu_free;
        } else {
            for (int64_t first = 0; first < m; first += B) {
                const int64_t b = (m - first < B) ? m - first : B;
                int32_t w = 0;
                for (int32_t j = 1; j < k; ++j)
                    if (free_at[j] < free_at[w]) w = j;
                const double start = free_at[w] > arrival[i] ? free_at[w] : arrival[i];
                free_at[w] = start + c[b];
                if (free_at[w] > done) done = free_at[w];
            }
        }
        latency[i] = done - arrival[i];
    }
}

void orc_two_tier_latencies(const double* arrival, const int64_t* size, int64_t n, int64_t tau, int64_t B,
                            const double* c, int32_t k, const double* g, double* latency) {
    double* free_at = (double*)malloc(sizeof(double) * (size_t)(k > 0 ? k : 1));
    orc_two_tier_run(arrival, size, n, tau, B, c, k, g, latency, free_at);
    free(free_at);
}

static int orc_two_tier_ok(const double* unit_arrival, const int64_t* size, int64_t n, int64_t tau, int64_t B,
                           const double* c, int32_t k, const double* g, double p, double sla, double rate,
                           double* arr, double* lat, double* free_at) {
    for (int64_t i = 0; i < n; ++i) arr[i] = unit_arrival[i] / rate;
    orc_two_tier_run(arr, size, n, tau, B, c, k, g, lat, free_at);
    return orc_percentile(lat, n, p) <= sla;
}

/* Latency-bounded throughput of the two tiers for a threshold tau: as orc_max_qps, with the
 * latencies of orc_two_tier_latencies.  The no-queueing check serves every query on an idle
 * system (each on its own, arrival 0). */
double orc_two_tier_max_qps(const double* unit_arrival, const int64_t* size, int64_t n, int64_t tau, int64_t B,
                            const double* c, int32_t k, const double* g, double p, double sla, int32_t iters) {
    if (n <= 0) return 0.0;
    double* arr = (double*)malloc(sizeof(double) * (size_t)n);
    double* lat = (double*)malloc(sizeof(double) * (size_t)n);
    double* free_at = (double*)malloc(sizeof(double) * (size_t)(k > 0 ? k : 1));
    const double zero = 0.0;
    for (int64_t i = 0; i < n; ++i) orc_two_tier_run(&zero, size + i, 1, tau, B, c, k, g, lat + i, free_at);
    double result = 0.0;
    if (orc_percentile(lat, n, p) <= sla) {
        double lo = 1.0, hi = 1.0;
#define OK(r) orc_two_tier_ok(unit_arrival, size, n, tau, B, c, k, g, p, sla, (r), arr, lat, free_at)
        if (OK(1.0)) {
            hi = 2.0;
            while (hi < 1e15 && OK(hi)) { lo = hi; hi *= 2.0; }
        } else {
            lo = 0.5;
            while (lo > 1e-15 && !OK(lo)) { hi = lo; lo *= 0.5; }
        }
        for (int32_t it = 0; it < iters; ++it) {
            const double mid = 0.5 * (lo + hi);
            if (OK(mid)) lo = mid; else hi = mid;
        }
#undef OK
        result = lo;
    }
    free(arr);
    free(lat);
    free(free_at);
    return result;
}

