// Query serving around the model forward: request service times, the single-device FIFO queue,
// latency-bounded throughput, the batch-size hill climb, an open-loop trace replay on the GPU, and
// the stream pool / throughput-mode entry point that keep several requests in flight.
//
// DeepRecSys paper: Section III-C (Poisson arrivals, query sizes), Section IV-A (a query is split
// into requests of a batch size), Section III-B (throughput is the query rate sustained under a
// p95 latency target), Section IV-C (the batch size is found by hill climbing on that rate).
// Everything here is host code; the replay and the throughput mode drive rec_model_forward.
#include <algorithm>
#include <chrono>
#include <cmath>
#include <functional>
#include <limits>
#include <new>
#include <thread>
#include <vector>

// REC_HOST_ONLY: build just the host-side functions (rec_sched_*) with a plain C++ compiler -- no HIP
// headers, no device calls -- so that they can run under the host sanitizers.
#ifdef REC_HOST_ONLY
#include "rec.h"
#else
#include "rec_common.h"
#endif

namespace {

const double kNaN = std::numeric_limits<double>::quiet_NaN();

// latencies of a FIFO single-server queue, written to lat; returns nothing (sizes checked by callers)
void fifo(const double* arrival, const double* service, int64_t n, double* lat) {
    double free_at = 0.0;                      // when the device becomes idle
    for (int64_t q = 0; q < n; ++q) {
        const double begin = (q == 0) ? arrival[q] : std::max(arrival[q], free_at);
        free_at = begin + service[q];
        lat[q] = free_at - arrival[q];
    }
}

double nearest_rank(std::vector<double>& v, double p) {
    const int64_t n = (int64_t)v.size();
    int64_t k = (int64_t)std::ceil(p * (double)n) - 1;
    k = std::min(std::max<int64_t>(k, 0), n - 1);
    std::nth_element(v.begin(), v.begin() + k, v.end());
    return v[k];
}

struct RateTest {
    const double* unit_arrival;
    const double* service;
    int64_t n;
    double p, sla;
    std::vector<double> arr, lat;
    bool operator()(double rate) {
        for (int64_t i = 0; i < n; ++i) arr[i] = unit_arrival[i] / rate;
        fifo(arr.data(), service, n, lat.data());
        return nearest_rank(lat, p) <= sla;    // nth_element reorders lat, which is rewritten next time
    }
};

// Two-tier queue: the accelerator is one FIFO server; CPU requests go, in arrival order, to the
// worker that frees up first (a min-heap of the workers' free times).
struct TwoTier {
    const int64_t* size;
    int64_t n, tau, batch;
    const double* c;
    int32_t k;
    const double* g;
    std::vector<double> heap;                  // scratch: k free times

    void run(const double* arrival, double* lat) {
        run_range(arrival, 0, n, lat);
    }
    // queries [first, last) on a system that starts idle; arrival/lat are indexed from `first`
    void run_range(const double* arrival, int64_t first, int64_t last, double* lat) {
        heap.assign((size_t)k, 0.0);           // all equal: already a heap
        double device_free = 0.0;
        for (int64_t q = first; q < last; ++q) {
            const double at = arrival[q - first];
            const int64_t m = size[q];
            double finished = at;
            if (m >= tau) {
                device_free = std::max(device_free, at) + g[m];
                finished = device_free;
            } else {
                for (int64_t left = m; left > 0; left -= batch) {
                    const int64_t b = std::min(left, batch);
                    std::pop_heap(heap.begin(), heap.end(), std::greater<double>());
                    const double end = std::max(heap.back(), at) + c[b];
                    heap.back() = end;
                    std::push_heap(heap.begin(), heap.end(), std::greater<double>());
                    finished = std::max(finished, end);
                }
            }
            lat[q - first] = finished - at;
        }
    }
};

bool two_tier_args_ok(const int64_t* size, int64_t n, int64_t tau, int64_t batch, const double* c, int32_t k,
                      const double* g, int64_t size_max) {
    if (!size || !c || !g || n < 0 || tau < 0 || batch < 1 || k < 1 || size_max < 0) return false;
    for (int64_t i = 0; i < n; ++i)
        if (size[i] < 0 || size[i] > size_max) return false;
    return true;
}

}  // namespace

#ifndef REC_HOST_ONLY
struct rec_stream_pool {
    std::vector<hipStream_t> streams;
};
#endif

extern "C" {

#ifndef REC_HOST_ONLY
rec_status rec_stream_pool_create(int32_t n_streams, rec_stream_pool** out) {
    if (!out) return REC_ERR_NULL;
    *out = nullptr;
    if (n_streams < 1 || n_streams > 16) return REC_ERR_BAD_SHAPE;
    rec_stream_pool* p = new (std::nothrow) rec_stream_pool;
    if (!p) return REC_ERR_DEVICE;
    for (int32_t i = 0; i < n_streams; ++i) {
        hipStream_t s = nullptr;
        if (hipStreamCreateWithFlags(&s, hipStreamNonBlocking) != hipSuccess) {
            rec_stream_pool_destroy(p);
            return REC_ERR_DEVICE;
        }
        p->streams.push_back(s);
    }
    *out = p;
    return REC_OK;
}

void rec_stream_pool_destroy(rec_stream_pool* pool) {
    if (!pool) return;
    for (hipStream_t s : pool->streams) {
        (void)hipStreamSynchronize(s);
        (void)hipStreamDestroy(s);
    }
    delete pool;
}

int32_t rec_stream_pool_size(const rec_stream_pool* pool) { return pool ? (int32_t)pool->streams.size() : 0; }

void* rec_stream_pool_stream(const rec_stream_pool* pool, int32_t i) {
    if (!pool || i < 0 || i >= (int32_t)pool->streams.size()) return nullptr;
    return pool->streams[(size_t)i];
}

rec_status rec_stream_pool_synchronize(const rec_stream_pool* pool) {
    if (!pool) return REC_ERR_NULL;
    for (hipStream_t s : pool->streams)
        if (hipStreamSynchronize(s) != hipSuccess) return REC_ERR_DEVICE;
    return REC_OK;
}

#endif  // REC_HOST_ONLY

double rec_sched_query_service(int64_t n, int64_t batch, const double* table) {
    if (n < 0 || batch < 1 || !table) return kNaN;
    const int64_t full = n / batch, rest = n % batch;
    double total = 0.0;
    for (int64_t k = 0; k < full; ++k) total += table[batch];   // added one by one, in request order
    if (rest) total += table[rest];
    return total;
}

rec_status rec_sched_fifo_latencies(const double* arrival, const double* service, int64_t n, double* latency) {
    if (n < 0) return REC_ERR_BAD_SHAPE;
    if (n == 0) return REC_OK;
    if (!arrival || !service || !latency) return REC_ERR_NULL;
    for (int64_t i = 1; i < n; ++i)
        if (arrival[i] < arrival[i - 1]) return REC_ERR_BAD_SHAPE;
    fifo(arrival, service, n, latency);
    return REC_OK;
}

double rec_sched_percentile(const double* x, int64_t n, double p) {
    if (!x || n < 1 || !(p > 0.0) || p > 1.0) return kNaN;
    std::vector<double> v(x, x + n);
    return nearest_rank(v, p);
}

double rec_sched_max_qps(const double* unit_arrival, const double* service, int64_t n, double p, double sla,
                         int32_t iters) {
    if (!unit_arrival || !service || n < 1 || !(p > 0.0) || p > 1.0 || iters < 0) return kNaN;
    {
        std::vector<double> s(service, service + n);
        if (nearest_rank(s, p) > sla) return 0.0;
    }
    RateTest ok{unit_arrival, service, n, p, sla, std::vector<double>((size_t)n), std::vector<double>((size_t)n)};
    double feasible, infeasible;
    if (ok(1.0)) {
        feasible = 1.0;
        infeasible = 2.0;
        while (infeasible < 1e15 && ok(infeasible)) {
            feasible = infeasible;
            infeasible *= 2.0;
        }
    } else {
        infeasible = 1.0;
        feasible = 0.5;
        while (feasible > 1e-15 && !ok(feasible)) {
            infeasible = feasible;
            feasible *= 0.5;
        }
    }
    for (int32_t k = 0; k < iters; ++k) {
        const double mid = 0.5 * (feasible + infeasible);
        if (ok(mid)) feasible = mid;
        else infeasible = mid;
    }
    return feasible;
}

rec_status rec_sched_two_tier_latencies(const double* arrival, const int64_t* size, int64_t n, int64_t tau,
                                        int64_t batch, const double* c, int32_t k, const double* g, int64_t size_max,
                                        double* latency) {
    if (n == 0) return REC_OK;
    if (!arrival || !latency || !size || !c || !g) return REC_ERR_NULL;
    if (!two_tier_args_ok(size, n, tau, batch, c, k, g, size_max)) return REC_ERR_BAD_SHAPE;
    for (int64_t i = 1; i < n; ++i)
        if (arrival[i] < arrival[i - 1]) return REC_ERR_BAD_SHAPE;
    TwoTier sim{size, n, tau, batch, c, k, g, {}};
    sim.run(arrival, latency);
    return REC_OK;
}

double rec_sched_two_tier_max_qps(const double* unit_arrival, const int64_t* size, int64_t n, int64_t tau, int64_t batch,
                                  const double* c, int32_t k, const double* g, int64_t size_max, double p, double sla,
                                  int32_t iters) {
    if (!unit_arrival || n < 1 || !(p > 0.0) || p > 1.0 || iters < 0) return kNaN;
    if (!two_tier_args_ok(size, n, tau, batch, c, k, g, size_max)) return kNaN;
    TwoTier sim{size, n, tau, batch, c, k, g, {}};
    std::vector<double> arr((size_t)n), lat((size_t)n);
    const double zero = 0.0;
    for (int64_t q = 0; q < n; ++q) sim.run_range(&zero, q, q + 1, &lat[(size_t)q]);   // every query alone on an idle system
    if (nearest_rank(lat, p) > sla) return 0.0;
    auto ok = [&](double rate) {
        for (int64_t i = 0; i < n; ++i) arr[(size_t)i] = unit_arrival[i] / rate;
        sim.run(arr.data(), lat.data());
        return nearest_rank(lat, p) <= sla;
    };
    double feasible, infeasible;
    if (ok(1.0)) {
        feasible = 1.0;
        infeasible = 2.0;
        while (infeasible < 1e15 && ok(infeasible)) {
            feasible = infeasible;
            infeasible *= 2.0;
        }
    } else {
        infeasible = 1.0;
        feasible = 0.5;
        while (feasible > 1e-15 && !ok(feasible)) {
            infeasible = feasible;
            feasible *= 0.5;
        }
    }
    for (int32_t it = 0; it < iters; ++it) {
        const double mid = 0.5 * (feasible + infeasible);
        if (ok(mid)) feasible = mid;
        else infeasible = mid;
    }
    return feasible;
}

int64_t rec_sched_hill_climb(const double* qps, int64_t n_candidates) {
    if (!qps || n_candidates < 1) return -1;
    int64_t keep = 0;
    for (int64_t next = 1; next < n_candidates; ++next) {
        if (qps[next] < qps[keep]) break;       // the rate degrades: stop climbing
        keep = next;
    }
    return keep;
}

#ifndef REC_HOST_ONLY

rec_status rec_model_forward_many(const rec_model* m, const rec_request* requests, float* const* prob, int64_t n,
                                  void* const* streams, void* const* workspaces, size_t workspace_bytes,
                                  int32_t n_streams) {
    if (n < 0 || n_streams < 1) return REC_ERR_BAD_SHAPE;
    if (n == 0) return REC_OK;
    if (!m || !requests || !prob || !streams || !workspaces) return REC_ERR_NULL;
    // requests of stream k: k, k + S, k + 2S, ... in order; returns the first failure on that stream
    auto run_stream = [&](int32_t k, int64_t* failed_at) {
        for (int64_t i = k; i < n; i += n_streams) {
            const rec_request& rq = requests[i];
            const rec_status st = rec_model_forward(m, rq.dense, rq.indices, rq.n_indices, rq.lengths, rq.B, prob[i],
                                                    workspaces[k], workspace_bytes, streams[k]);
            if (st != REC_OK) {
                *failed_at = i;
                return st;
            }
        }
        *failed_at = n;
        return REC_OK;
    };
    // A forward is five to seven launches of a few microseconds of host time each; with short
    // batches the device outruns one enqueuing thread, so a long list gets a thread per stream.
    if (n_streams == 1 || n < 8 * (int64_t)n_streams) {
        for (int64_t i = 0; i < n; ++i) {
            const rec_request& rq = requests[i];
            const int32_t k = (int32_t)(i % n_streams);
            const rec_status st = rec_model_forward(m, rq.dense, rq.indices, rq.n_indices, rq.lengths, rq.B, prob[i],
                                                    workspaces[k], workspace_bytes, streams[k]);
            if (st != REC_OK) return st;
        }
        return REC_OK;
    }
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) return REC_ERR_DEVICE;
    std::vector<rec_status> status((size_t)n_streams, REC_OK);
    std::vector<int64_t> failed_at((size_t)n_streams, n);
    std::vector<std::thread> workers;
    for (int32_t k = 1; k < n_streams; ++k)
        workers.emplace_back([&, k]() {
            if (hipSetDevice(device) != hipSuccess) {
                status[(size_t)k] = REC_ERR_DEVICE;
                failed_at[(size_t)k] = k;
                return;
            }
            status[(size_t)k] = run_stream(k, &failed_at[(size_t)k]);
        });
    status[0] = run_stream(0, &failed_at[0]);
    for (std::thread& t : workers) t.join();
    // report the failure of the lowest-numbered request
    int32_t worst = 0;
    for (int32_t k = 1; k < n_streams; ++k)
        if (failed_at[(size_t)k] < failed_at[(size_t)worst]) worst = k;
    return status[(size_t)worst];
}

rec_status rec_serve_trace(const rec_model* m, const rec_request* requests, const int64_t* query_first,
                           const double* arrival_s, int64_t n_queries, float* prob, void* workspace,
                           size_t workspace_bytes, void* stream, double* latency_s) {
    return rec_serve_trace_many(m, requests, query_first, arrival_s, n_queries, &prob, &workspace, workspace_bytes, &stream,
                                1, 0, latency_s);
}

rec_status rec_serve_trace_many(const rec_model* m, const rec_request* requests, const int64_t* query_first,
                                const double* arrival_s, int64_t n_queries, float* const* prob,
                                void* const* workspaces, size_t workspace_bytes, void* const* streams,
                                int32_t n_streams, int32_t spread_requests, double* latency_s) {
    if (n_queries < 0 || n_streams < 1) return REC_ERR_BAD_SHAPE;
    if (n_queries == 0) return REC_OK;
    if (!m || !requests || !query_first || !arrival_s || !latency_s || !prob || !workspaces || !streams) return REC_ERR_NULL;
    for (int32_t k = 0; k < n_streams; ++k)
        if (!prob[k]) return REC_ERR_NULL;
    int64_t n_marks = 0;
    for (int64_t q = 0; q < n_queries; ++q) {
        const int64_t n_req = query_first[q + 1] - query_first[q];
        if (n_req < 0 || arrival_s[q] < 0.0) return REC_ERR_BAD_SHAPE;
        if (q > 0 && arrival_s[q] < arrival_s[q - 1]) return REC_ERR_BAD_SHAPE;
        n_marks += spread_requests ? std::max<int64_t>(1, std::min<int64_t>(n_req, n_streams)) : 1;
    }
    // A query is complete when the last of its requests on every stream it used is: one event per
    // (query, stream used), recorded behind that request.  origin[k] is time zero as stream k sees it.
    struct Mark {
        int32_t stream;
        hipEvent_t event;
    };
    std::vector<Mark> marks((size_t)n_marks, Mark{0, nullptr});
    std::vector<int64_t> mark_first((size_t)n_queries + 1, 0);
    std::vector<hipEvent_t> origin((size_t)n_streams, nullptr);
    auto cleanup = [&]() {
        for (Mark& k : marks)
            if (k.event) (void)hipEventDestroy(k.event);
        for (hipEvent_t e : origin)
            if (e) (void)hipEventDestroy(e);
    };
    auto sync_all = [&]() {
        bool ok = true;
        for (int32_t k = 0; k < n_streams; ++k) ok = (hipStreamSynchronize(static_cast<hipStream_t>(streams[k])) == hipSuccess) && ok;
        return ok;
    };
    for (Mark& k : marks)
        if (hipEventCreate(&k.event) != hipSuccess) {
            cleanup();
            return REC_ERR_DEVICE;
        }
    for (auto& e : origin)
        if (hipEventCreate(&e) != hipSuccess) {
            cleanup();
            return REC_ERR_DEVICE;
        }
    // time zero: every stream is idle and its origin event has just completed, so device
    // timestamps measured from it and host time measured from t0 share an origin to within the
    // latency of the synchronisation
    bool ok = sync_all();
    for (int32_t k = 0; k < n_streams && ok; ++k)
        ok = hipEventRecord(origin[(size_t)k], static_cast<hipStream_t>(streams[k])) == hipSuccess;
    ok = ok && sync_all();
    if (!ok) {
        cleanup();
        return REC_ERR_DEVICE;
    }
    const auto t0 = std::chrono::steady_clock::now();
    rec_status st = REC_OK;
    int64_t next_mark = 0;
    int64_t turn = 0;                                     // round-robin position over the streams
    std::vector<char> used((size_t)n_streams, 0);
    for (int64_t q = 0; q < n_queries && st == REC_OK; ++q) {
        mark_first[(size_t)q] = next_mark;
        while (std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count() < arrival_s[q]) {
        }
        std::fill(used.begin(), used.end(), 0);
        const int32_t home = (int32_t)(turn % n_streams);
        for (int64_t r = query_first[q]; r < query_first[q + 1] && st == REC_OK; ++r) {
            const int32_t k = spread_requests ? (int32_t)(turn++ % n_streams) : home;
            const rec_request& rq = requests[r];
            st = rec_model_forward(m, rq.dense, rq.indices, rq.n_indices, rq.lengths, rq.B, prob[k], workspaces[k],
                                   workspace_bytes, streams[k]);
            used[(size_t)k] = 1;
        }
        if (!spread_requests) ++turn;
        if (query_first[q + 1] == query_first[q]) used[(size_t)home] = 1;      // an empty query still gets a time stamp
        for (int32_t k = 0; k < n_streams && st == REC_OK; ++k) {
            if (!used[(size_t)k]) continue;
            Mark& mk = marks[(size_t)next_mark++];
            mk.stream = k;
            if (hipEventRecord(mk.event, static_cast<hipStream_t>(streams[k])) != hipSuccess) st = REC_ERR_DEVICE;
        }
    }
    mark_first[(size_t)n_queries] = next_mark;
    if (!sync_all() && st == REC_OK) st = REC_ERR_DEVICE;
    if (st == REC_OK) {
        for (int64_t q = 0; q < n_queries && st == REC_OK; ++q) {
            double finished = 0.0;
            for (int64_t i = mark_first[(size_t)q]; i < mark_first[(size_t)q + 1]; ++i) {
                float ms = 0.f;
                if (hipEventElapsedTime(&ms, origin[(size_t)marks[(size_t)i].stream], marks[(size_t)i].event) != hipSuccess) {
                    st = REC_ERR_DEVICE;
                    break;
                }
                finished = std::max(finished, (double)ms * 1e-3);
            }
            latency_s[q] = finished - arrival_s[q];
        }
    }
    cleanup();
    return st;
}

#endif  // REC_HOST_ONLY

}  // extern "C"
