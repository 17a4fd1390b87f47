"""Puts a synthetic workload (see ``synth``) on the device as a ``rec.Model`` plus
batches.  Input plumbing only: generation, host-to-device copies and the one-off
bf16 conversion of the weights (done by the library's own converter)."""
from __future__ import annotations

import numpy as np
import torch

from . import rec, synth


def device_tables(cfg: synth.Config, device="cuda", seed: int = synth.MASTER_SEED) -> rec.Tables:
    return rec.Tables([synth.table_full_torch(cfg, t, device, seed) for t in range(cfg.T)])


def device_mlp(params: synth.MLPParams, bf16: bool, device="cuda"):
    W = [torch.from_numpy(w).to(device) for w in params.W]
    b = [torch.from_numpy(v).to(device) for v in params.b]
    if bf16:
        W = [rec.f32_to_bf16(w) for w in W]
    return W, b


def device_model(cfg: synth.Config, device="cuda", seed: int = synth.MASTER_SEED, tables: rec.Tables | None = None,
                 caller_padded_weights: bool = False):
    tables = tables if tables is not None else device_tables(cfg, device, seed)
    Wb, bb = device_mlp(synth.mlp_params(cfg.bottom, 0, seed), cfg.bf16, device)
    Wt, bt = device_mlp(synth.mlp_params(cfg.top, 1, seed), cfg.bf16, device)
    return rec.Model(tables, Wb, bb, Wt, bt, rec.BF16 if cfg.bf16 else rec.F32,
                     interaction=rec.INTERACT_CONCAT if cfg.interaction == "concat" else rec.INTERACT_DOT,
                     dense_features=cfg.F, caller_padded_weights=caller_padded_weights)


class DeviceBatch:
    def __init__(self, batch: synth.Batch, device="cuda"):
        self.B = batch.B
        self.dense = torch.from_numpy(batch.dense).to(device)
        self.indices = torch.from_numpy(batch.indices).to(device)
        self.lengths = torch.from_numpy(batch.lengths).to(device)
        self.n_indices = int(batch.indices.size)


def slice_batch(batch: synth.Batch, T: int, start: int, count: int) -> synth.Batch:
    """Samples start..start+count-1 of a batch, as a batch of its own (table-major bags)."""
    B = batch.B
    off = np.concatenate([[0], np.cumsum(batch.lengths, dtype=np.int64)])
    lens, idx = [], []
    for t in range(T):
        lo, hi = t * B + start, t * B + start + count
        lens.append(batch.lengths[lo:hi])
        idx.append(batch.indices[off[lo]:off[hi]])
    return synth.Batch(count, batch.dense[start:start + count].copy(),
                       np.concatenate(lens).astype(np.int32), np.concatenate(idx).astype(np.int32))
