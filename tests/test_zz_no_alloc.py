"""rec_sls_forward_static (the pooling entry point that takes no workspace and allocates nothing)
against rec_sls_forward, through the C ABI: same bits, on two calls in a row, the second smaller."""
import numpy as np
import pytest
import torch

from paper_2001_02772_amd import rec, synth

pytestmark = pytest.mark.gpu


def _case(cfg, k, B):
    b = synth.BatchGenerator(cfg).batch(k, B=B)
    return torch.from_numpy(b.indices).cuda(), torch.from_numpy(b.lengths).cuda()


def test_static_scratch_pooling_matches_workspace_pooling_twice():
    rec.lib()
    cfg = synth.CONFIGS["rmc1"].replace(R=20_000, T=6, len_lo=0, len_hi=90)
    tables = rec.Tables([torch.from_numpy(synth.table_full(cfg, t)).cuda() for t in range(cfg.T)])
    for k, B in ((0, 700), (1, 130)):                      # the second call is the smaller one
        idx, lens = _case(cfg, k, B)
        want = rec.sls_forward(tables, idx, lens, B)
        got = rec.sls_forward_static(tables, idx, lens, B)
        torch.cuda.synchronize()
        assert got.shape == want.shape == (B, cfg.T, cfg.D)
        assert torch.equal(got, want), f"call {k}: static-scratch pooling differs from rec_sls_forward"
        # strided output, as the model uses it
        V = cfg.T + 1
        a = torch.zeros((B, V, cfg.D), dtype=torch.float32, device="cuda")
        rec.sls_forward_static(tables, idx, lens, B, out=a[:, 1:, :], out_stride_b=V * cfg.D, out_stride_t=cfg.D)
        torch.cuda.synchronize()
        assert torch.equal(a[:, 1:, :], want) and float(a[:, 0, :].abs().max()) == 0.0


def test_static_scratch_pooling_rejects_what_does_not_fit():
    rec.lib()
    cfg = synth.CONFIGS["tiny"]
    tables = rec.Tables([torch.zeros((16, 8), dtype=torch.float32, device="cuda") for _ in range(4)])
    B = rec.SLS_STATIC_MAX_BAGS // 4                        # T*B + 1 is one more than the array holds
    lens = torch.zeros(4 * B, dtype=torch.int32, device="cuda")
    idx = torch.zeros(0, dtype=torch.int32, device="cuda")
    with pytest.raises(rec.RecError) as e:
        rec.sls_forward_static(tables, idx, lens, B)
    assert e.value.status == rec.ERR_WORKSPACE
    out = rec.sls_forward_static(tables, idx, lens[: 4 * (B - 1)], B - 1)    # the largest that fits: all bags empty -> zeros
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0
