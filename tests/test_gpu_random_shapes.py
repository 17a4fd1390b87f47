"""Seeded random shapes through the FC planner and the whole model, against the oracle: the
planner has many regimes (fused runs, tiled layers, the large-tile bf16 kernel, k splits, the
scan riding in a fused launch or not, padded first predictor layer, short-bag pooling), and
hand-picked cases only cover the boundaries somebody thought of.  Every shape is inside the
limits the header documents."""
import numpy as np
import pytest
import torch

import oracle
from paper_2001_02772_amd import synth
from parity_util import TOL_BF16, TOL_F32, assert_close, oracle_forward

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rec():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2001_02772_amd import rec as _rec
    _rec.lib()
    return _rec


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _widths(r, n_layers, lo=1, hi=700):
    # mix of tiny, unaligned, narrow and wide layers
    pool = [1, 2, 3, 7, 8, 13, 16, 31, 32, 33, 64, 87, 100, 128, 255, 256, 257, 384, 512, 513, 640]
    return [int(r.choice(pool)) if r.random() < 0.7 else int(r.integers(lo, hi + 1)) for _ in range(n_layers + 1)]


@pytest.mark.parametrize("seed", range(24))
def test_mlp_random_stack(rec, seed):
    r = np.random.default_rng(1000 + seed)
    bf16 = bool(seed % 2)
    n_layers = int(r.integers(1, 6))
    widths = _widths(r, n_layers)
    B = int(r.choice([1, 5, 16, 17, 63, 100, 256, 300, 1024]))
    final = int(r.choice([0, 1, 2]))
    p = synth.mlp_params(tuple(widths), 0, 77 + seed)
    x = r.normal(size=(B, widths[0])).astype(np.float32)
    print(f"[random mlp] seed {seed}: widths {widths}, B {B}, bf16 {bf16}, final act {final}", flush=True)
    W = [dev(w) for w in p.W]
    if bf16:
        W = [rec.f32_to_bf16(w) for w in W]
    got = rec.mlp_forward(W, [dev(b) for b in p.b], dev(x), rec.ACT_RELU, final,
                          wdtype=rec.BF16 if bf16 else rec.F32).cpu().numpy()
    want = oracle.mlp(x, p.W, p.b, rec.ACT_RELU, final, bf16=bf16)
    assert_close(got, want, TOL_BF16 if bf16 else TOL_F32, f"random stack {widths} B={B}")


@pytest.mark.parametrize("seed", range(16))
def test_model_random_config(rec, seed):
    from paper_2001_02772_amd import workload
    r = np.random.default_rng(2000 + seed)
    concat = seed % 4 == 3
    T = int(r.integers(1, 28))
    D = int(r.choice([4, 8, 16, 32, 48, 64, 128]))
    F = int(r.choice([1, 4, 13, 64, 200])) if not concat else int(r.choice([4, 16, 64]))
    B = int(r.choice([1, 3, 16, 40, 129, 257]))
    R = int(r.integers(5, 400))
    lo, hi = [(0, 0), (1, 1), (0, 3), (0, 40), (20, 20), (60, 100)][int(r.integers(0, 6))]
    if concat:
        no_stack = bool(r.integers(0, 2))
        X = F if no_stack else int(r.choice([4, 8, 32]))
        bottom = (F,) if no_stack else (F, int(r.choice([16, 33, 64])), X)
        top = (X + T * D, int(r.choice([16, 64, 100, 300])), 1)
    else:
        bottom = (F, int(r.choice([8, 64, 256])), D)
        top = (D + (T + 1) * T // 2, int(r.choice([16, 64, 100, 512])), int(r.choice([8, 32])), 1)
    cfg = synth.Config(f"random-{seed}", B, F, T, R, D, lo, hi, "uniform" if seed % 2 else "zipf", "normal", bottom, top,
                       bf16=bool(seed % 3 == 0), interaction="concat" if concat else "dot")
    synth.check_config(cfg)
    print(f"[random model] seed {seed}: {cfg}", flush=True)
    tables = [synth.table_full(cfg, t) for t in range(cfg.T)]
    model = workload.device_model(cfg, tables=rec.Tables([dev(t) for t in tables]))
    batch = synth.BatchGenerator(cfg).batch(seed)
    db = workload.DeviceBatch(batch)
    got = model.forward(db.dense, db.indices, db.lengths, B).cpu().numpy()
    want = oracle_forward(cfg, tables, batch)
    assert_close(got, want, TOL_BF16 if cfg.bf16 else TOL_F32, f"random model {seed}")
