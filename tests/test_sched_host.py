"""The library's host-side serving functions against the oracle: same inputs, results equal
bit for bit (they are sequences of IEEE double additions, divisions and comparisons in a
fixed order, so nothing but equality is expected).  CPU only: no kernel is launched."""
import math

import numpy as np
import pytest

import oracle
from paper_2001_02772_amd import synth


@pytest.fixture(scope="module")
def rec():
    from paper_2001_02772_amd import rec as _rec
    _rec.lib()
    return _rec


def service_table(B, seed):
    r = np.random.default_rng(seed)
    t = 40e-6 + np.cumsum(r.uniform(0.0, 0.3e-6, B + 1))     # increasing, launch floor + per-item cost
    t[0] = 0.0
    return t


def test_query_service_matches_oracle(rec):
    t = service_table(1024, 1)
    for B in (1, 3, 16, 64, 256, 1000, 1024):
        for n in list(range(0, 70)) + [255, 256, 257, 999, 1000, 1001, 4096, 5000]:
            assert rec.sched_query_service(n, B, t) == oracle.query_service(n, B, t)
    assert math.isnan(rec.sched_query_service(-1, 4, t))
    assert math.isnan(rec.sched_query_service(4, 0, t))


def test_fifo_matches_oracle(rec):
    r = np.random.default_rng(2)
    for n, load in [(1, 0.5), (2, 0.9), (500, 0.5), (500, 0.95), (500, 1.3)]:
        a = np.cumsum(r.exponential(1.0, n))
        s = r.exponential(load, n)
        assert np.array_equal(rec.sched_fifo_latencies(a, s), oracle.fifo_latencies(a, s))
    assert rec.sched_fifo_latencies([], []).size == 0
    with pytest.raises(rec.RecError):
        rec.sched_fifo_latencies([1.0, 0.5], [1.0, 1.0])          # arrivals out of order


def test_percentile_matches_oracle(rec):
    r = np.random.default_rng(3)
    for n in (1, 2, 19, 20, 21, 100, 1001):
        x = r.normal(size=n)
        x[: n // 3] = np.round(x[: n // 3])                       # ties
        for p in (0.01, 0.5, 0.95, 0.99, 1.0):
            assert rec.sched_percentile(x, p) == oracle.percentile(x, p)
    assert math.isnan(rec.sched_percentile([1.0], 0.0))
    assert math.isnan(rec.sched_percentile([1.0], 1.5))
    assert math.isnan(rec.sched_percentile([], 0.5))


def test_max_qps_and_hill_climb_match_oracle(rec):
    n = 2000
    sizes = synth.lognormal_query_sizes(synth.MASTER_SEED, n)
    unit = synth.unit_poisson_arrivals(synth.MASTER_SEED, n)
    t = service_table(1024, 4)
    cands = [1, 2, 4, 8, 16, 32, 64, 128, 256, 512, 1024]
    for sla in (1e-5, 1.5e-3, 3e-3, 10e-3):
        got, want = [], []
        for B in cands:
            svc = np.array([oracle.query_service(int(q), B, t) for q in sizes])
            got.append(rec.sched_max_qps(unit, svc, 0.95, sla, 40))
            want.append(oracle.max_qps(unit, svc, 0.95, sla, 40))
        assert got == want
        assert rec.sched_hill_climb(got) == oracle.hill_climb(np.array(want))
    assert rec.sched_max_qps(unit, np.full(n, 1.0), 0.95, 0.5, 40) == 0.0
    for q in ([1.0], [1.0, 2.0, 3.0], [1.0, 2.0, 2.0, 5.0], [3.0, 1.0, 9.0], [1.0, 2.0, 1.5, 4.0]):
        assert rec.sched_hill_climb(q) == oracle.hill_climb(np.array(q))
    assert rec.sched_hill_climb([]) == -1


def test_two_tier_matches_oracle(rec):
    r = np.random.default_rng(8)
    n, B = 600, 16
    c = np.concatenate([[0.0], 2e-3 + 1e-4 * np.arange(1, B + 1)])
    g = np.concatenate([[0.0], 3e-4 + 2e-7 * np.arange(1, 1001)])
    sizes = synth.lognormal_query_sizes(synth.MASTER_SEED, n)
    unit = synth.unit_poisson_arrivals(synth.MASTER_SEED, n)
    for tau in (1, 2, 17, 100, 400, 1001):
        for k in (1, 3, 16):
            for rate in (20.0, 300.0, 5000.0):
                a = unit / rate
                assert np.array_equal(rec.sched_two_tier_latencies(a, sizes, tau, B, c, k, g),
                                      oracle.two_tier_latencies(a, sizes, tau, B, c, k, g)), (tau, k, rate)
    qps_p, qps_o = [], []
    for tau in (1, 2, 4, 8, 16, 32, 64, 128, 256, 512, 1001):
        qps_p.append(rec.sched_two_tier_max_qps(unit, sizes, tau, B, c, 16, g, 0.95, 0.05))
        qps_o.append(oracle.two_tier_max_qps(unit, sizes, tau, B, c, 16, g, 0.95, 0.05))
    assert qps_p == qps_o
    assert rec.sched_hill_climb(qps_p) == oracle.hill_climb(np.array(qps_o))
    assert rec.sched_two_tier_max_qps(unit, sizes, 1001, B, c, 16, g, 0.95, 1e-4) == 0.0        # idle system misses it
    # argument errors
    assert math.isnan(rec.sched_two_tier_max_qps(unit, sizes, 4, B, c, 0, g, 0.95, 0.05))        # no workers
    assert math.isnan(rec.sched_two_tier_max_qps(unit, sizes, 4, B, c, 2, g[:500], 0.95, 0.05))  # a size beyond g
    with pytest.raises(rec.RecError):
        rec.sched_two_tier_latencies([1.0, 0.5], [3, 3], 4, B, c, 2, g)
