"""Parity at the full benchmark sizes, in the launch configuration the benchmark
times.  The oracle runs the whole batch too: it is given only the table rows the
batch touches (regenerated from the counter-based stream), so every output
element is compared."""
import numpy as np
import pytest
import torch

from paper_2001_02772_amd import synth
from parity_util import TOL_BF16, TOL_F32, assert_close, compact_tables, oracle_forward

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rec():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2001_02772_amd import rec as _rec
    _rec.lib()
    return _rec


@pytest.mark.parametrize("name", ["rmc1", "rmc2", "rmc2-uniform", "rmc3", "wnd"])
def test_full_size_model_and_sls(rec, name):
    import oracle
    from paper_2001_02772_amd import workload
    oracle.set_threads(16)
    cfg = synth.CONFIGS[name]
    print(f"[full-size] {name}: building model", flush=True)
    model = workload.device_model(cfg)
    # the device tables hold the same values the oracle's row generator produces
    probe = np.array([0, 1, cfg.R // 2, cfg.R - 1])
    assert np.array_equal(model.tables.tensors[cfg.T - 1][torch.from_numpy(probe).cuda()].cpu().numpy(),
                          synth.table_rows(cfg, cfg.T - 1, probe))
    batch = synth.BatchGenerator(cfg).batch(1)
    db = workload.DeviceBatch(batch)
    print(f"[full-size] {name}: validate + forward, N={db.n_indices}", flush=True)
    assert rec.sls_validate([cfg.R] * cfg.T, db.indices, db.lengths, cfg.B) == (rec.OK, 0, -1)
    got = model.forward(db.dense, db.indices, db.lengths, cfg.B).cpu().numpy()
    sls = rec.sls_forward(model.tables, db.indices, db.lengths, cfg.B).cpu().numpy()
    print(f"[full-size] {name}: oracle", flush=True)
    small_tables, idx = compact_tables(cfg, batch)
    assert np.array_equal(rec.sls_offsets(db.lengths).cpu().numpy(), oracle.offsets(batch.lengths))
    E, _, aabs = oracle.sls(small_tables, idx, batch.lengths, cfg.B, extra=True)
    assert_close(sls, E, TOL_F32, f"{name} SLS")
    L = batch.lengths.reshape(cfg.T, cfg.B).T[:, :, None]
    assert np.all(np.abs(sls.astype(np.float64) - E) <= (L + 1) * 2.0**-24 * aabs + 1e-30)
    want = oracle_forward(cfg, small_tables, batch, indices=idx)
    e = assert_close(got, want, TOL_BF16 if cfg.bf16 else TOL_F32, f"{name} model")
    print(f"[full-size] {name}: max rel err {e:.3e}", flush=True)
    oracle.set_threads(1)


@pytest.mark.parametrize("name", ["rmc2", "rmc3"])
def test_full_size_throughput_mode(rec, name):
    """The launch configuration the benchmark times: requests enqueued by one
    rec_model_forward_many call over a four-stream pool.  Every output of every request equals
    the single-stream forward bit for bit, and one batch is checked against the oracle in full."""
    import oracle
    from paper_2001_02772_amd import workload
    pool = rec.StreamPool(4)
    cfg = synth.CONFIGS[name]
    print(f"[full-size many] {name}: building model", flush=True)
    model = workload.device_model(cfg)
    gen = synth.BatchGenerator(cfg)
    batches = [gen.batch(k) for k in (1, 2, 3)]
    dbs = [workload.DeviceBatch(b) for b in batches]
    single = [model.forward(d.dense, d.indices, d.lengths, cfg.B).clone() for d in dbs]
    reqs = [dbs[i % 3] for i in range(36)]                       # 36 >= 8 * 4: one enqueuing thread per stream
    probs = [torch.zeros(cfg.B, dtype=torch.float32, device="cuda") for _ in reqs]
    torch.cuda.synchronize()
    print(f"[full-size many] {name}: forward_many", flush=True)
    rec.ForwardMany(model, reqs, probs, pool.streams).launch()
    pool.synchronize()
    for i, p in enumerate(probs):
        assert torch.equal(p, single[i % 3]), i
    print(f"[full-size many] {name}: oracle", flush=True)
    oracle.set_threads(16)
    small_tables, idx = compact_tables(cfg, batches[1])
    want = oracle_forward(cfg, small_tables, batches[1], indices=idx)
    oracle.set_threads(1)
    assert_close(probs[1].cpu().numpy(), want, TOL_BF16 if cfg.bf16 else TOL_F32, f"{name} forward_many")
