/* rec.h -- C ABI of librec: batched forward inference of a DLRM-style
 * recommendation model on one MI355X (gfx950).
 *
 * The model is the generalised architecture of Figure 2 / Section II-A of the
 * DeepRecSys paper with the DLRM-RMC parameters of Table I: dense features go
 * through a stack of fully-connected layers ("Dense-FC"), each sparse feature
 * indexes rows of its embedding table and the rows are sum-pooled, the dense
 * and pooled vectors are combined by a feature interaction, and a second FC
 * stack ("Predict-FC") turns the result into one click-through probability per
 * user-item pair.
 *
 * Conventions
 *   - Pointers marked DEV are device pointers owned by the caller; pointers
 *     marked HOST are host pointers read before the call returns.  The compute
 *     calls never allocate or free device memory; scratch comes in through the
 *     `workspace` arguments (256-byte aligned, at least *_workspace_bytes()).
 *     The only calls that create device-side resources are rec_model_create
 *     (at most one buffer, see there) and rec_stream_pool_create (streams).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     The compute calls only enqueue work and return; the synchronous ones say
 *     so: rec_sls_validate, rec_model_create, rec_stream_pool_synchronize /
 *     _destroy, rec_serve_trace and rec_serve_trace_many.
 *   - Errors that the host can see (null pointer, bad shape, small workspace)
 *     are returned before anything is launched.  Errors that depend on device
 *     data (negative length, lengths not summing to n_indices, index out of
 *     range) are detected ONLY by rec_sls_validate; the forward calls do not
 *     check device data and their behaviour on such input is undefined.
 *   - Batch size 0 and empty bags are legal.
 *   - Bags are table-major: bag t*B + b holds the lookups of sample b into
 *     table t; `indices` is the concatenation of all bags in that order.
 *   - Results are deterministic: no atomics, fixed reduction orders.
 *   - Calls on different streams with disjoint workspaces and outputs may
 *     overlap; a model handle is immutable after creation.
 */
#ifndef REC_H
#define REC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    REC_OK = 0,
    REC_ERR_NULL = 1,              /* a required pointer is NULL */
    REC_ERR_BAD_SHAPE = 2,         /* negative / inconsistent sizes or strides */
    REC_ERR_NEGATIVE_LENGTH = 3,   /* validate: some bag length < 0 */
    REC_ERR_LENGTHS_MISMATCH = 4,  /* validate: sum(lengths) != n_indices */
    REC_ERR_INDEX_RANGE = 5,       /* validate: some index outside [0, rows[t]) */
    REC_ERR_WORKSPACE = 6,         /* workspace NULL, misaligned or too small */
    REC_ERR_UNSUPPORTED = 7,       /* e.g. D not a multiple of 4, rows[t] > 2^31-1 */
    REC_ERR_DEVICE = 8             /* a HIP call or kernel launch failed */
} rec_status;

typedef enum { REC_F32 = 0, REC_BF16 = 1 } rec_dtype;
typedef enum { REC_ACT_NONE = 0, REC_ACT_RELU = 1, REC_ACT_SIGMOID = 2 } rec_act;

/* Static, NUL-terminated name of a status code. */
const char* rec_status_string(rec_status s);

/* ---- query splitting (Section IV-A: a query of n candidate items is divided
 * into requests of a chosen batch size) ------------------------------------
 * Consecutive slices: floor(n/batch) of size `batch`, then one of n mod batch
 * if that is non-zero.  Writes (start, count) pairs to the HOST arrays and
 * returns the number of slices; with start == count == NULL it only counts.
 * Returns -1 if n < 0 or batch < 1. */
int64_t rec_split_query(int64_t n, int64_t batch, int64_t* start, int64_t* count);

/* ---- embedding lookup + sum pooling (Section II-A, "Embedding Table Access";
 * Table I, pooling = Sum) ----------------------------------------------------
 *   E[b][t][:] = sum_{k < lengths[t*B+b]} Table_t[ indices[off(t,b) + k] ][:]
 * for all T tables in one launch; duplicates count with multiplicity, an
 * empty bag gives zeros.  Sums are fp32.
 *
 *   tables      DEV array of T DEV pointers, table t is fp32 [rows[t]][D]
 *               row-major, base 16-byte aligned (256-byte recommended)
 *   rows        HOST int64[T], each in [1, 2^31-1]
 *   D           multiple of 4, 4 <= D <= 256
 *   indices     DEV int32 [n_indices]
 *   lengths     DEV int32 [T*B]
 *   out         DEV fp32; element (b,t,d) at out[b*out_stride_b + t*out_stride_t + d]
 *               (strides in floats, multiples of 4, out 16-byte aligned), so the
 *               result can land in slots 1..T of a [B][T+1][D] interaction buffer
 *   workspace   DEV, >= rec_sls_workspace_bytes(T, B); receives the offsets
 */
size_t rec_sls_workspace_bytes(int32_t T, int32_t B);
rec_status rec_sls_forward(const float* const* tables, const int64_t* rows, int32_t T, int32_t D,
                           const int32_t* indices, int64_t n_indices, const int32_t* lengths,
                           int32_t B, float* out, int64_t out_stride_b, int64_t out_stride_t,
                           void* workspace, size_t workspace_bytes, void* stream);

/* The same pooling with the bag offsets already computed (rec_sls_offsets):
 * offsets DEV int64 [T*B + 1], bag i covers indices[offsets[i] .. offsets[i+1]).
 * Launches the gather-and-pool kernel alone; needs no workspace. */
rec_status rec_sls_forward_offsets(const float* const* tables, const int64_t* rows, int32_t T, int32_t D,
                                   const int32_t* indices, int64_t n_indices, const int64_t* offsets,
                                   int32_t B, float* out, int64_t out_stride_b, int64_t out_stride_t,
                                   void* stream);

/* rec_sls_forward for callers that cannot hand over or allocate scratch memory: code running
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation calls.  Same
 * arguments and result as rec_sls_forward minus the workspace: the bag offsets go to an array that
 * is part of the library's device image (REC_SLS_STATIC_MAX_BAGS 64-bit offsets, 2 MiB, one copy
 * per GPU the library runs on, held until the process ends).  Calls no allocation routine.
 * Returns REC_ERR_WORKSPACE, and launches nothing, when T*B + 1 > REC_SLS_STATIC_MAX_BAGS.
 * Every call on a GPU uses that GPU's one array: calls that overlap on the same GPU (different
 * streams or threads) race; calls on one stream do not.  Nothing needs clearing between calls (each
 * call writes every offset before reading it). */
#define REC_SLS_STATIC_MAX_BAGS 262144
rec_status rec_sls_forward_static(const float* const* tables, const int64_t* rows, int32_t T, int32_t D,
                                  const int32_t* indices, int64_t n_indices, const int32_t* lengths,
                                  int32_t B, float* out, int64_t out_stride_b, int64_t out_stride_t,
                                  void* stream);

/* Exclusive prefix sum of bag lengths (the offsets used above):
 * offsets[0] = 0, offsets[i+1] = offsets[i] + lengths[i].
 * lengths DEV int32 [n_bags]; offsets DEV int64 [n_bags + 1], 16-byte aligned. */
rec_status rec_sls_offsets(const int32_t* lengths, int64_t n_bags, int64_t* offsets, void* stream);

/* Input check for the sparse side; SYNCHRONOUS (waits for `stream`, reads a
 * few words back).  In this order: any length < 0 -> REC_ERR_NEGATIVE_LENGTH;
 * 64-bit sum of lengths != n_indices -> REC_ERR_LENGTHS_MISMATCH; any index of
 * table t outside [0, rows[t]) -> REC_ERR_INDEX_RANGE with *n_bad = how many
 * and *first_bad = flat position of the first (else 0 and -1).
 * n_bad / first_bad are HOST pointers (may be NULL).  Same workspace size as
 * rec_sls_forward. */
rec_status rec_sls_validate(const int64_t* rows, int32_t T, const int32_t* indices,
                            int64_t n_indices, const int32_t* lengths, int32_t B,
                            int64_t* n_bad, int64_t* first_bad,
                            void* workspace, size_t workspace_bytes, void* stream);

/* ---- fully-connected stacks (Section II-A, "Features" and "Product
 * Ranking"; widths per Table I) -----------------------------------------------
 *   y = act_L( ... act_1( x W_1^T + b_1 ) ... W_L^T + b_L )
 * Hidden layers use hidden_act, the last layer final_act.
 *
 *   W        HOST array of n_layers DEV pointers; W[l] is [widths[l+1]][widths[l]]
 *            row-major in `wdtype` (REC_F32: float; REC_BF16: bfloat16 bit patterns)
 *   bias     HOST array of n_layers DEV pointers to fp32 [widths[l+1]]
 *   widths   HOST int32 [n_layers + 1], all >= 1
 *   x        DEV fp32 [B][widths[0]], row stride ldx floats
 *   y        DEV fp32 [B][widths[n_layers]], row stride ldy floats
 * REC_F32: fp32 operands, fp32 accumulation.  REC_BF16: the activations entering
 * each layer and the weights are bf16 (round to nearest even), products are
 * accumulated in fp32, bias and activation are applied in fp32, y is fp32. */
size_t rec_mlp_workspace_bytes(const int32_t* widths, int32_t n_layers, int32_t B, rec_dtype wdtype);
rec_status rec_mlp_forward(const void* const* W, const float* const* bias, const int32_t* widths,
                           int32_t n_layers, rec_dtype wdtype, rec_act hidden_act, rec_act final_act,
                           const float* x, int64_t ldx, float* y, int64_t ldy, int32_t B,
                           void* workspace, size_t workspace_bytes, void* stream);

/* fp32 -> bfloat16 (round to nearest even, NaN stays NaN), for preparing
 * REC_BF16 weights.  src DEV fp32 [n], dst DEV uint16 [n]. */
rec_status rec_f32_to_bf16(const float* src, uint16_t* dst, int64_t n, void* stream);

/* ---- feature interaction (Section II-A, "Feature Interaction": the outputs of
 * the dense and sparse sides are combined before the predictor stack) ---------
 * Pairwise dot products: vecs DEV fp32 [B][V][D] (slot 0 = dense-stack output,
 * slots 1..V-1 = pooled embeddings), and for each sample
 *   out[b] = [ vecs[b][0][0..D) , <vecs[b][i], vecs[b][j]> for i = 1..V-1, j = 0..i-1 ]
 * i.e. slot 0 copied, then the strict lower triangle of V V^T row by row.
 * out DEV fp32 [B][D + V(V-1)/2], row stride ldo floats.  1 <= V <= 128,
 * D multiple of 4, 4 <= D <= 256. */
rec_status rec_interact(const float* vecs, int32_t B, int32_t V, int32_t D,
                        float* out, int64_t ldo, void* stream);

/* ---- whole model (Figure 2) ------------------------------------------------
 * REC_INTERACT_DOT (the DLRM rows of Table I): offsets -> SLS into slots 1..T of
 * [B][T+1][D]; bottom stack (ReLU after every layer) into slot 0; interaction; top
 * stack (ReLU on hidden layers, sigmoid on the 1-wide last layer) -> one probability
 * per sample.
 * REC_INTERACT_CONCAT (the "Concat" rows of Table I, NCF / Wide&Deep; Section II-A):
 * the top stack's input is [ x | E_0 | ... | E_{T-1} ], x = bottom stack output, or the
 * dense features themselves when n_bottom = 0 (bottom_widths = {F}, bottom_W/b unused);
 * E_t = pooled embedding of table t.  x's width must be a multiple of 4.
 * The handle BORROWS every pointer in the descriptor: DEV memory must stay
 * alive and unchanged while the handle is used; HOST arrays are copied.
 *
 * Padded weights.  The dot interaction's width D + T(T+1)/2 is rarely a multiple of what
 * the FC kernels load at a time, so the model runs the first top layer on a copy of its
 * weights with zero-padded rows (rec_model_padded_weight_bytes() says how large; 0 = none
 * needed).  Two ways to provide it:
 *   - desc.padded_weights = NULL: rec_model_create allocates the copy, fills it and
 *     synchronises the device once; rec_model_destroy frees it.
 *   - desc.padded_weights = a DEV buffer of at least that many bytes, 256-byte aligned,
 *     owned by the caller: rec_model_create is then host-only (no device allocation, no
 *     device work, no synchronisation) and the caller enqueues rec_model_prepare() once
 *     before the first forward. */
typedef enum { REC_INTERACT_DOT = 0, REC_INTERACT_CONCAT = 1 } rec_interaction;

typedef struct {
    int32_t T;                       /* embedding tables, 1 <= T <= 127 */
    int32_t D;                       /* embedding dim = bottom stack output width */
    const float* const* tables;      /* DEV array of T DEV pointers (as rec_sls_forward) */
    const int64_t* rows;             /* HOST int64[T] */
    int32_t n_bottom;                /* bottom layers */
    const int32_t* bottom_widths;    /* HOST [n_bottom+1]; [0] = dense features F, last = D */
    const void* const* bottom_W;     /* HOST array of DEV pointers (as rec_mlp_forward) */
    const float* const* bottom_b;
    int32_t n_top;                   /* top layers */
    const int32_t* top_widths;       /* HOST [n_top+1]; [0] = D + T(T+1)/2, last = 1 */
    const void* const* top_W;
    const float* const* top_b;
    rec_dtype mlp_dtype;             /* REC_F32 or REC_BF16, both stacks */
    rec_interaction interaction;     /* REC_INTERACT_DOT: bottom_widths last = D, top_widths[0] = D + T(T+1)/2;
                                        REC_INTERACT_CONCAT: top_widths[0] = bottom_widths last + T*D */
    void* padded_weights;            /* DEV, caller-owned, or NULL (see "Padded weights" above) */
    size_t padded_weights_bytes;     /* size of that buffer */
} rec_model_desc;

typedef struct rec_model rec_model;

/* Bytes of the padded copy of the first top layer's weights this descriptor needs (0: none).
 * HOST only; looks at the widths and dtype, not at the pointers. */
size_t rec_model_padded_weight_bytes(const rec_model_desc* desc);
rec_status rec_model_create(const rec_model_desc* desc, rec_model** out);
/* Fills the caller-provided padded-weights buffer (one small launch on `stream`, no allocation,
 * no synchronisation).  Needed once, before the first forward, only when desc.padded_weights was
 * given and rec_model_padded_weight_bytes() > 0; otherwise a no-op.  Until then the forward
 * calls return REC_ERR_BAD_SHAPE.  Call it from one thread, before the handle is shared. */
rec_status rec_model_prepare(rec_model* m, void* stream);
void rec_model_destroy(rec_model* m);
size_t rec_model_workspace_bytes(const rec_model* m, int32_t B_max);

/*   dense    DEV fp32 [B][F] contiguous (16-byte aligned when the model has no bottom stack)
 *   indices  DEV int32 [n_indices];  lengths DEV int32 [T*B]
 *   prob     DEV fp32 [B]
 *   workspace >= rec_model_workspace_bytes(m, B) */
rec_status rec_model_forward(const rec_model* m, const float* dense, const int32_t* indices,
                             int64_t n_indices, const int32_t* lengths, int32_t B, float* prob,
                             void* workspace, size_t workspace_bytes, void* stream);

/* ---- query serving and batch-size tuning -------------------------------------
 * Section III-C: queries arrive as a Poisson process and carry a number of candidate items
 * (the query size); Section IV-A: a query is split into requests of the chosen batch size;
 * Section III-B: the figure of merit is the query rate sustained while the p95 query latency
 * stays under a target; Section IV-C: the batch size is tuned by hill climbing on that rate.
 * All arrays in this group are HOST arrays of doubles (seconds, queries/s). */

/* Time to serve a query of n items as floor(n/batch) requests of `batch` items plus one of
 * n mod batch items, one after another: table[b] = seconds for one request of b items,
 * b = 1..batch (table[0] unused).  NaN if n < 0, batch < 1 or table is NULL. */
double rec_sched_query_service(int64_t n, int64_t batch, const double* table);

/* One device serving queries first-come-first-served: query i starts at max(arrival[i],
 * finish of query i-1) and takes service[i]; latency[i] = finish - arrival[i].  Arrivals must be
 * non-decreasing. */
rec_status rec_sched_fifo_latencies(const double* arrival, const double* service, int64_t n, double* latency);

/* Nearest-rank percentile: the smallest sample v with at least a fraction p of the samples
 * <= v, i.e. sorted[ceil(p*n) - 1]; p in (0, 1].  NaN if n < 1 or p out of range. */
double rec_sched_percentile(const double* x, int64_t n, double p);

/* Latency-bounded throughput: the largest rate r (queries/s) for which the p-th percentile of
 * the FIFO latencies with arrivals unit_arrival[i] / r stays <= sla, where unit_arrival are the
 * arrival times of a rate-1 Poisson process.  0 if the percentile of `service` alone exceeds sla.
 * Search: r = 1 is tested; feasible -> double until infeasible (cap 1e15), infeasible -> halve
 * until feasible (floor 1e-15); then `iters` bisection steps; the feasible end is returned.
 * NaN on bad arguments. */
double rec_sched_max_qps(const double* unit_arrival, const double* service, int64_t n, double p, double sla,
                         int32_t iters);

/* Hill climb over candidate batch sizes in increasing order (first = unit batch size):
 * qps[i] = achievable rate with candidate i.  Moves to the next candidate until the rate
 * degrades: stops at the first step that lowers it (steps that leave it unchanged are taken, so
 * the climb crosses batch sizes that all miss the latency target).  Returns the index kept,
 * -1 if n_candidates < 1 or qps is NULL. */
int64_t rec_sched_hill_climb(const double* qps, int64_t n_candidates);

/* Two tiers (Section IV-B, "Leverage parallelism with specialized hardware"; Section IV-C,
 * second hill climb): queries of tau items or more go whole to the accelerator -- one device,
 * first come first served, g[m] seconds for a query of m items, transfer included -- and the
 * others are cut into requests of `batch` items that run on k identical CPU workers: requests are
 * handed out in arrival order, each to the worker that is free first, c[b] seconds for a request
 * of b items; a query is done when its last request is.  tau = 1 sends everything to the
 * accelerator (where the paper's climb starts), tau above the largest size sends nothing.
 * These two calls are the scheduler's queueing model only: nothing here runs a model on the CPU.
 * HOST arrays: arrival (non-decreasing) / unit_arrival, size int64 [n] (each >= 0), c [batch+1],
 * g [max size + 1], latency [n].  size_max = length of g minus 1 (sizes above it are an error). */
rec_status rec_sched_two_tier_latencies(const double* arrival, const int64_t* size, int64_t n, int64_t tau,
                                        int64_t batch, const double* c, int32_t k, const double* g, int64_t size_max,
                                        double* latency);

/* Largest rate r with the p-th percentile of the two-tier latencies (arrivals unit_arrival / r)
 * <= sla; search as rec_sched_max_qps; 0 if the percentile on an idle system (every query served
 * alone) already exceeds sla.  NaN on bad arguments. */
double rec_sched_two_tier_max_qps(const double* unit_arrival, const int64_t* size, int64_t n, int64_t tau, int64_t batch,
                                  const double* c, int32_t k, const double* g, int64_t size_max, double p, double sla,
                                  int32_t iters);

/* One request = one rec_model_forward call: inputs as for rec_model_forward (all DEV). */
typedef struct {
    const float* dense;
    const int32_t* indices;
    int64_t n_indices;
    const int32_t* lengths;
    int32_t B;
} rec_request;

/* A set of streams owned by the library for requests that may overlap on the device: default
 * priority, not synchronised with the null stream (the caller orders them against whatever
 * produced the inputs, e.g. by synchronising the device once after set-up).  1 <= n <= 16.
 * Streams that share one of the runtime's few hardware queues do not overlap, and which
 * streams share is settled when they are created: create the pool before the process creates
 * other streams or runs other device work (measured: a pool created first spreads over 4 queues,
 * one created after a framework's set-up behaved like 2 streams). */
typedef struct rec_stream_pool rec_stream_pool;
rec_status rec_stream_pool_create(int32_t n_streams, rec_stream_pool** out);
void rec_stream_pool_destroy(rec_stream_pool* pool);                 /* waits for the streams' work first */
int32_t rec_stream_pool_size(const rec_stream_pool* pool);
void* rec_stream_pool_stream(const rec_stream_pool* pool, int32_t i); /* NULL if i is out of range */
rec_status rec_stream_pool_synchronize(const rec_stream_pool* pool);

/* Throughput mode (Section III-B counts completed work per second, not the latency of one
 * request): request i runs on streams[i % n_streams] with workspaces[i % n_streams] and writes
 * prob[i] (DEV fp32 [requests[i].B]).  Requests that share a stream run in order; requests on
 * different streams overlap on the device, so the short latency-bound kernels of one request
 * fill the gaps of another.  ASYNCHRONOUS on every stream; the caller orders the streams
 * against whatever produced the inputs and synchronises them before reading prob.
 * HOST: requests [n], prob [n] (array of DEV pointers), streams [n_streams], workspaces
 * [n_streams] (DEV, each >= workspace_bytes >= rec_model_workspace_bytes(m, max B)).
 * A long list (n >= 8 n_streams) is enqueued by one host thread per stream.  A request that
 * fails ends its stream's list; the status of the lowest-numbered failing request is returned. */
rec_status rec_model_forward_many(const rec_model* m, const rec_request* requests, float* const* prob, int64_t n,
                                  void* const* streams, void* const* workspaces, size_t workspace_bytes,
                                  int32_t n_streams);

/* Open-loop replay of a query trace on one device (SYNCHRONOUS, busy-waits on the host clock):
 * query q, made of requests[query_first[q] .. query_first[q+1]), is submitted to `stream` when
 * the host clock reaches arrival_s[q] (seconds from the start of the call, non-decreasing) and
 * never before; requests run in order.  latency_s[q] = completion of the query's last request
 * (device timestamp) - arrival_s[q].  prob: DEV fp32 [max request B], overwritten by every
 * request; workspace >= rec_model_workspace_bytes(m, max request B).  HOST: requests,
 * query_first [n_queries + 1], arrival_s, latency_s [n_queries]. */
rec_status rec_serve_trace(const rec_model* m, const rec_request* requests, const int64_t* query_first,
                           const double* arrival_s, int64_t n_queries, float* prob, void* workspace,
                           size_t workspace_bytes, void* stream, double* latency_s);

/* rec_serve_trace over several streams, each with its own prob[k] (DEV fp32 [max request B]) and
 * workspaces[k].  spread_requests = 0: query q runs on streams[q % n_streams], its requests in
 * order on that stream; queries on different streams overlap on the device.  spread_requests != 0:
 * the requests themselves are dealt round-robin over the streams, so the requests of one query run
 * side by side -- the request-level parallelism of Section IV-A with streams in the place of
 * cores -- and the query is complete when the last of them is.  Everything else as
 * rec_serve_trace (which is this call with one stream). */
rec_status rec_serve_trace_many(const rec_model* m, const rec_request* requests, const int64_t* query_first,
                                const double* arrival_s, int64_t n_queries, float* const* prob,
                                void* const* workspaces, size_t workspace_bytes, void* const* streams,
                                int32_t n_streams, int32_t spread_requests, double* latency_s);

#ifdef __cplusplus
}
#endif
#endif /* REC_H */
