"""Open-loop trace replay on the GPU: the probabilities it leaves are those of the plain
forward (checked against the oracle), and the measured latencies obey what a FIFO device
must obey whatever its speed.  Timing itself is not asserted beyond loose physical bounds."""
import numpy as np
import pytest
import torch

from paper_2001_02772_amd import synth
from parity_util import TOL_F32, assert_close, compact_tables, oracle_forward

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def setup():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2001_02772_amd import rec, workload
    rec.lib()
    cfg = synth.CONFIGS["tiny"]
    model = workload.device_model(cfg)
    batch = synth.BatchGenerator(cfg).batch(0)
    return rec, workload, cfg, model, batch


def split(rec, workload, cfg, batch, sizes, B):
    """queries of the given sizes taken from consecutive samples of `batch`, each cut into requests of <= B"""
    queries, start = [], 0
    for n in sizes:
        reqs, done = [], 0
        while done < n:
            c = min(B, n - done)
            reqs.append(workload.DeviceBatch(workload.slice_batch(batch, cfg.T, start + done, c)))
            done += c
        queries.append(reqs)
        start += n
    return queries


def test_replay_results_and_fifo_properties(setup):
    rec, workload, cfg, model, batch = setup
    sizes = [5, 1, 9, 4, 7, 3]
    assert sum(sizes) <= cfg.B
    queries = split(rec, workload, cfg, batch, sizes, 4)
    print("[serving] burst replay", flush=True)
    lat = rec.serve_trace(model, queries, np.zeros(len(sizes)))
    # every query arrives at time zero: completions are ordered and each one waits for all before it
    assert np.all(lat > 0) and np.all(np.diff(lat) > 0)
    assert lat[-1] < 1.0
    print("[serving] spaced replay", flush=True)
    gap = 5e-3
    arr = np.arange(len(sizes)) * gap
    lat2 = rec.serve_trace(model, queries, arr)
    # widely spaced arrivals: nothing queues, nothing is submitted early, every latency is one service time
    assert np.all(lat2 > 0) and np.all(lat2 < gap)
    # the last request of the last query is what the output buffer holds
    last = queries[-1][-1]
    prob = torch.empty(4, dtype=torch.float32, device="cuda")
    ws = model.workspace(4)
    import ctypes as C
    reqs = (rec._Request * 1)(rec._Request(rec._ptr(last.dense), rec._ptr(last.indices), last.indices.numel(),
                                           rec._ptr(last.lengths), last.B))
    first = np.array([0, 1], dtype=np.int64)
    a = np.zeros(1)
    out = np.zeros(1)
    st = rec.lib().rec_serve_trace(model._h, C.addressof(reqs), first.ctypes.data, a.ctypes.data, 1, rec._ptr(prob),
                                   rec._ptr(ws), ws.numel(), rec._stream(), out.ctypes.data)
    assert st == rec.OK and out[0] > 0
    hb = workload.slice_batch(batch, cfg.T, sum(sizes) - last.B, last.B)
    sub = cfg.replace(B=last.B)
    small, idx = compact_tables(sub, hb)
    want = oracle_forward(sub, small, hb, indices=idx)
    assert_close(prob[: last.B].cpu().numpy(), want, TOL_F32, "replayed request")
    assert np.array_equal(prob[: last.B].cpu().numpy(),
                          model.forward(last.dense, last.indices, last.lengths, last.B).cpu().numpy())


def test_replay_rejects_bad_traces(setup):
    rec, workload, cfg, model, batch = setup
    queries = split(rec, workload, cfg, batch, [2, 2], 2)
    with pytest.raises(rec.RecError):
        rec.serve_trace(model, queries, np.array([1e-3, 0.0]))       # arrivals out of order
    with pytest.raises(rec.RecError):
        rec.serve_trace(model, queries, np.array([-1.0, 0.0]))
    assert rec.serve_trace(model, [], np.zeros(0)).size == 0


def test_forward_many_matches_single_forward(setup):
    rec, workload, cfg, model, batch = setup
    sizes = [5, 1, 16, 4, 7, 3, 9, 12, 2]
    reqs, start = [], 0
    for n in sizes:
        reqs.append(workload.DeviceBatch(workload.slice_batch(batch, cfg.T, start, n)))
        start += n
    want = [model.forward(r.dense, r.indices, r.lengths, r.B).clone() for r in reqs]
    torch.cuda.synchronize()
    for n_streams in (1, 3):
        pool = rec.StreamPool(n_streams)
        streams = pool.streams
        assert len(streams) == n_streams and all(s.cuda_stream for s in streams)
        probs = [torch.zeros(r.B, dtype=torch.float32, device="cuda") for r in reqs]
        torch.cuda.synchronize()
        fm = rec.ForwardMany(model, reqs, probs, streams)
        fm.launch()
        pool.synchronize()
        for p, w in zip(probs, want):
            assert torch.equal(p, w)
    # a long list takes the path with one enqueuing host thread per stream
    long_reqs, long_want = reqs * 4, want * 4
    pool = rec.StreamPool(3)
    assert len(long_reqs) >= 8 * 3
    long_probs = [torch.zeros(r.B, dtype=torch.float32, device="cuda") for r in long_reqs]
    torch.cuda.synchronize()
    for _ in range(2):
        rec.ForwardMany(model, long_reqs, long_probs, pool.streams).launch()
    pool.synchronize()
    for p, w in zip(long_probs, long_want):
        assert torch.equal(p, w)
    # against the oracle as well
    sub = cfg.replace(B=sum(sizes))
    hb = workload.slice_batch(batch, cfg.T, 0, sum(sizes))
    small, idx = compact_tables(sub, hb)
    assert_close(torch.cat(probs).cpu().numpy(), oracle_forward(sub, small, hb, indices=idx), TOL_F32, "forward_many")
    with pytest.raises(rec.RecError):
        bad = rec.ForwardMany(model, reqs, probs, streams)
        bad.ws_bytes = 16                                            # workspace too small
        bad.launch()
    torch.cuda.synchronize()
    with pytest.raises(rec.RecError):
        rec.StreamPool(0)
    with pytest.raises(rec.RecError):
        rec.StreamPool(17)


def test_replay_over_stream_pool(setup):
    rec, workload, cfg, model, batch = setup
    sizes = [5, 1, 9, 4, 7, 3, 6, 2]
    queries = split(rec, workload, cfg, batch, sizes, 4)
    pool = rec.StreamPool(3)
    tr = rec.ServeTrace(model, queries, pool.streams)
    print("[serving] pool burst replay", flush=True)
    lat = tr.run(np.zeros(len(sizes)))
    assert np.all(lat > 0) and lat.max() < 1.0
    for k in range(3):                       # queries that share a stream complete in order
        assert np.all(np.diff(lat[k::3]) > 0)
    print("[serving] pool spaced replay", flush=True)
    gap = 5e-3
    lat2 = tr.run(np.arange(len(sizes)) * gap)
    assert np.all(lat2 > 0) and np.all(lat2 < gap)
    # requests dealt over the streams: a query is complete when the slowest of its requests is
    spread = rec.ServeTrace(model, queries, pool.streams, spread_requests=True)
    lat3 = spread.run(np.zeros(len(sizes)))
    assert np.all(lat3 > 0) and lat3.max() < 1.0
    lat4 = spread.run(np.arange(len(sizes)) * gap)
    assert np.all(lat4 > 0) and np.all(lat4 < gap)
    # each stream's output buffer holds the last request of the last query that ran on it
    for k in range(3):
        q = max(i for i in range(len(sizes)) if i % 3 == k)
        last = queries[q][-1]
        want = model.forward(last.dense, last.indices, last.lengths, last.B)
        assert torch.equal(tr.prob[k][: last.B], want)
