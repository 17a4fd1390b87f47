"""Helpers for the GPU-vs-oracle parity tests (CPU side only: NumPy + the oracle)."""
import numpy as np

import oracle
from paper_2001_02772_amd import synth

TOL_F32 = 1e-5     # max relative error, fp32 paths
TOL_BF16 = 2e-2    # max relative error, bf16-operand FC outputs


def rel_err(got, want):
    """max |g-o| / max(|o|, s), s = RMS of the oracle tensor (relative error is
    undefined at ReLU zeros and cancelling sums, so small values are measured
    against the tensor's own scale)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    if want.size == 0:
        return 0.0
    s = float(np.sqrt(np.mean(want * want)))
    den = np.maximum(np.abs(want), s if s > 0 else 1.0)
    return float(np.max(np.abs(got - want) / den))


def assert_close(got, want, tol, what=""):
    assert np.all(np.isfinite(np.asarray(got))), f"{what}: non-finite values"
    e = rel_err(got, want)
    assert e <= tol, f"{what}: max relative error {e:.3e} > {tol:.1e}"
    return e


def compact_tables(cfg, batch, seed=synth.MASTER_SEED):
    return synth.compact_tables(cfg, batch, seed)


def oracle_forward(cfg, tables, batch, indices=None, seed=synth.MASTER_SEED):
    pb, pt = synth.mlp_params(cfg.bottom, 0, seed), synth.mlp_params(cfg.top, 1, seed)
    st, p = oracle.model_forward(tables, pb.W, pb.b, pt.W, pt.b, batch.dense,
                                 batch.indices if indices is None else indices, batch.lengths, bf16=cfg.bf16,
                                 concat=cfg.interaction == "concat")
    assert st == oracle.OK
    return p
