"""The seeded input generators: determinism, random access, distributions."""
import numpy as np
import torch

from paper_2001_02772_amd import synth


def test_splitmix64_published_vectors():
    # first outputs of SplitMix64 started at state 1234567 (reference values that
    # accompany the published generator)
    key = np.uint64(1234567)
    c = np.arange(3, dtype=np.uint64)
    with np.errstate(over="ignore"):
        out = synth._mix(key + synth._GAMMA * (c + np.uint64(1)))
    assert out.tolist() == [6457827717110365317, 3203168211198807973, 9817491932198370423]


def test_random_access_equals_sequential():
    a = synth.draws(5, 77, 1000, 64)
    b = synth.draws_at(5, 77, np.arange(1000, 1064))
    assert np.array_equal(a, b)
    assert not np.array_equal(a, synth.draws(5, 78, 1000, 64))
    assert not np.array_equal(a, synth.draws(6, 77, 1000, 64))


def test_table_rows_match_full_table_and_torch():
    cfg = synth.CONFIGS["tiny"]
    full = synth.table_full(cfg, 3, chunk_rows=999)
    assert full.shape == (10_000, 32) and full.dtype == np.float32
    rows = np.array([0, 17, 9999, 17])
    assert np.array_equal(synth.table_rows(cfg, 3, rows), full[rows])
    assert np.array_equal(synth.table_full_torch(cfg, 3, "cpu", chunk_rows=777).numpy(), full)
    assert full.min() >= -0.05 and full.max() < 0.05 and abs(full.mean()) < 1e-3
    assert not np.array_equal(full, synth.table_full(cfg, 4))


def test_batches_are_reproducible_and_shaped():
    cfg = synth.CONFIGS["rmc1"].replace(R=5000, B=32)
    g = synth.BatchGenerator(cfg)
    b0, b0again, b1 = g.batch(0), synth.BatchGenerator(cfg).batch(0), g.batch(1)
    assert np.array_equal(b0.indices, b0again.indices) and np.array_equal(b0.dense, b0again.dense)
    assert not np.array_equal(b0.lengths, b1.lengths)
    assert b0.dense.shape == (32, 13) and b0.dense.dtype == np.float32
    assert b0.lengths.shape == (cfg.T * 32,) and b0.lengths.dtype == np.int32
    assert b0.lengths.min() >= 60 and b0.lengths.max() <= 100
    assert b0.indices.size == b0.lengths.sum() and b0.indices.dtype == np.int32
    assert b0.indices.min() >= 0 and b0.indices.max() < 5000
    assert 0 <= b0.dense.min() and b0.dense.max() < 1
    # a short batch of the same stream
    assert g.batch(3, B=5).dense.shape == (5, 13)


def test_zipf_is_skewed_and_permuted():
    cfg = synth.CONFIGS["rmc2"].replace(R=20_000, B=64, T=2)
    g = synth.BatchGenerator(cfg)
    b = g.batch(0)
    n0 = int(b.lengths[:64].sum())
    idx0 = b.indices[:n0]
    cdf = synth.zipf_cdf(20_000, 1.05)
    # share of lookups that hit the 100 most popular ranks, vs the law
    hot_rows = g.perm(0)[:100]
    share = np.isin(idx0, hot_rows).mean()
    assert abs(share - cdf[99]) < 0.05
    assert sorted(g.perm(0).tolist()) == list(range(20_000))
    assert not np.array_equal(g.perm(0), g.perm(1))
    assert abs(cdf[-1] - 1.0) < 1e-12 and np.all(np.diff(cdf) > 0)


def test_normal_and_lognormal():
    z = synth.normal_f32(1, synth.stream_id(synth.K_DENSE), 0, 200_000)
    assert abs(z.mean()) < 0.01 and abs(z.std() - 1) < 0.01
    q = synth.lognormal_query_sizes(synth.MASTER_SEED, 2000)
    assert q.min() >= 1 and q.max() <= 1000 and q.dtype == np.int64
    assert 100 < q.mean() < 190               # exp(4.5 + 0.5) = 148 before clipping
    assert np.array_equal(q, synth.lognormal_query_sizes(synth.MASTER_SEED, 2000))


def test_configs_match_declared_shapes():
    c = synth.CONFIGS
    assert (c["tiny"].V, c["tiny"].P, c["tiny"].top[0]) == (9, 36, 68)
    assert (c["rmc1"].V, c["rmc1"].P, c["rmc1"].top[0]) == (11, 55, 87)
    assert (c["rmc2"].V, c["rmc2"].P, c["rmc2"].top[0]) == (41, 820, 884)
    assert (c["rmc3"].V, c["rmc3"].P, c["rmc3"].top[0]) == (11, 55, 87) and c["rmc3"].bf16
    p = synth.mlp_params(c["tiny"].bottom, 0)
    assert [w.shape for w in p.W] == [(64, 13), (32, 64)] and [b.shape for b in p.b] == [(64,), (32,)]
