"""Pins for the oracle's query-serving and hill-climbing functions: a hand-worked queue,
closed forms of the deterministic queue, an independent event-driven simulation, NumPy's
percentile, brute force.  CPU only."""
import math

import numpy as np

import oracle
from paper_2001_02772_amd import synth

rng = np.random.default_rng(3)


def test_fifo_and_service_hand_example(golden):
    g = golden("fifo_hand_example.txt")
    lat = oracle.fifo_latencies(g["arrival"], g["service"])
    assert lat.tolist() == g["latency"]
    assert (np.array(g["arrival"]) + lat).tolist() == g["finish"]
    assert oracle.query_service(int(g["query_items"][0]), int(g["batch"][0]), g["table"]) == g["query_service"][0]


def test_query_service_closed_forms():
    t = np.arange(0, 65, dtype=np.float64) ** 0.5          # any table
    for n in range(0, 200):
        for B in (1, 7, 16, 64):
            want = (n // B) * t[B] + (t[n % B] if n % B else 0.0)
            assert math.isclose(oracle.query_service(n, B, t), want, rel_tol=1e-12, abs_tol=0)
    # one request when the query fits
    assert oracle.query_service(5, 64, t) == t[5]


def test_fifo_deterministic_queue_closed_form():
    n = 50
    for d, s in [(2.0, 1.5), (2.0, 2.0), (1.0, 1.25)]:
        a = np.arange(n) * d
        lat = oracle.fifo_latencies(a, np.full(n, s))
        want = np.full(n, s) if s <= d else s + np.arange(n) * (s - d)
        assert np.allclose(lat, want, rtol=1e-12, atol=1e-12)


def test_fifo_vs_event_driven_simulation():
    n = 300
    a = np.cumsum(rng.exponential(1.0, n))
    s = rng.exponential(0.8, n)
    # independent formulation: walk a clock through arrival / departure events with an explicit queue
    clock, queue, busy_until, finish, i = 0.0, [], 0.0, np.zeros(n), 0
    serving = None
    while i < n or queue or serving is not None:
        next_arr = a[i] if i < n else math.inf
        next_dep = busy_until if serving is not None else math.inf
        if next_arr <= next_dep:
            clock = next_arr
            queue.append(i)
            i += 1
        else:
            clock = next_dep
            finish[serving] = clock
            serving = None
        if serving is None and queue:
            serving = queue.pop(0)
            busy_until = clock + s[serving]
    lat = oracle.fifo_latencies(a, s)
    assert np.allclose(lat, finish - a, rtol=1e-12, atol=1e-12)
    assert np.all(lat >= s - 1e-9)                           # never faster than its own service time
    # work conservation: the device is never idle while a query waits
    assert math.isclose((a + lat)[-1], max((a + lat)[-2], a[-1]) + s[-1], rel_tol=1e-12)


def test_percentile_nearest_rank():
    assert oracle.percentile(np.arange(1, 21.0), 0.95) == 19.0
    assert oracle.percentile(np.arange(1, 21.0), 1.0) == 20.0
    assert oracle.percentile([5.0], 0.95) == 5.0
    x = rng.normal(size=1001)
    for p in (0.5, 0.95, 0.99):
        assert oracle.percentile(x, p) == np.sort(x)[math.ceil(p * x.size) - 1]
        assert oracle.percentile(x, p) == np.percentile(x, 100 * p, method="inverted_cdf")


def test_max_qps_closed_form_deterministic():
    # evenly spaced unit arrivals, constant service s: no queue up to rate 1/s, beyond it query i
    # waits i*(s - 1/rate); with k = ceil(p n) - 1 the bound s + k (s - 1/rate) <= sla gives the rate
    n, s, p, sla = 200, 0.01, 0.95, 0.05
    unit = np.arange(1, n + 1, dtype=np.float64)
    k = math.ceil(p * n) - 1
    want = 1.0 / (s - (sla - s) / k)
    got = oracle.max_qps(unit, np.full(n, s), p, sla, iters=60)
    assert math.isclose(got, want, rel_tol=1e-9)
    assert got > 1.0 / s                                      # some queueing is tolerated by the target
    # a target below the service time cannot be met at any rate
    assert oracle.max_qps(unit, np.full(n, s), p, 0.5 * s) == 0.0
    # the answer is feasible and a slightly higher rate is not
    lat = oracle.fifo_latencies(unit / got, np.full(n, s))
    assert oracle.percentile(lat, p) <= sla
    lat = oracle.fifo_latencies(unit / (got * 1.001), np.full(n, s))
    assert oracle.percentile(lat, p) > sla


def test_max_qps_poisson_is_feasible_boundary_and_monotone_in_sla():
    n = 2000
    unit = synth.unit_poisson_arrivals(7, n)
    sizes = synth.lognormal_query_sizes(7, n)
    service = sizes * 2e-6 + 30e-6
    prev = 0.0
    assert oracle.max_qps(unit, service, 0.95, 0.5e-3) == 0.0     # p95 of the bare service times is 0.97 ms
    for sla in (1.5e-3, 3e-3, 10e-3):
        q = oracle.max_qps(unit, service, 0.95, sla)
        assert q >= prev
        prev = q
        assert oracle.percentile(oracle.fifo_latencies(unit / q, service), 0.95) <= sla
        assert oracle.percentile(oracle.fifo_latencies(unit / (q * 1.01), service), 0.95) > sla
    assert prev < 1.0 / service.mean()                        # never above saturation


def test_hill_climb_rule():
    assert oracle.hill_climb([1.0]) == 0
    assert oracle.hill_climb([1, 2, 3, 4]) == 3               # keeps improving to the end
    assert oracle.hill_climb([1, 2, 3, 2, 9]) == 2            # stops at the first degradation
    assert oracle.hill_climb([5, 4, 9]) == 0
    assert oracle.hill_climb([1, 2, 2, 3]) == 3               # a tie is not a degradation
    assert oracle.hill_climb([0, 0, 0, 5, 9, 7]) == 4         # batch sizes that miss the target: keep climbing
    assert oracle.hill_climb([5, 5, 5]) == 2
    for _ in range(50):                                       # unimodal sequences: the arg max
        q = rng.uniform(size=8)
        peak = rng.integers(0, 8)
        q = np.concatenate([np.sort(q[:peak + 1]), np.sort(q[peak + 1:])[::-1] * q[:peak + 1].max() * 0.99])
        assert oracle.hill_climb(q) == int(np.argmax(q))


def test_unit_poisson_arrivals():
    a = synth.unit_poisson_arrivals(11, 200_000)
    gaps = np.diff(a)
    assert np.all(gaps > 0) and abs(gaps.mean() - 1) < 0.01 and abs(gaps.std() - 1) < 0.01
    assert np.array_equal(a, synth.unit_poisson_arrivals(11, 200_000))
