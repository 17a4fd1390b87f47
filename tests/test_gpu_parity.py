"""GPU parity: every entry point of the C ABI against the CPU oracle, element by
element on the same seeded inputs.  Integer work (offsets, validator counts and
positions, bf16 bit patterns, query splits) must match bit for bit; fp32 results
within 1e-5, bf16-operand FC outputs within 2e-2 (relative, see rel_err)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2001_02772_amd import synth
from parity_util import TOL_BF16, TOL_F32, assert_close, compact_tables, oracle_forward, rel_err

pytestmark = pytest.mark.gpu

rng = np.random.default_rng(11)


@pytest.fixture(scope="module")
def rec():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2001_02772_amd import rec as _rec
    _rec.lib()
    return _rec


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _bags(T, B, R, lo, hi):
    lengths = rng.integers(lo, hi + 1, size=T * B).astype(np.int32)
    indices = rng.integers(0, R, size=int(lengths.sum())).astype(np.int32)
    return indices, lengths


# ------------------------------------------------------------------ integer work

@pytest.mark.parametrize("n", [0, 1, 63, 64, 4095, 4096, 4097, 40960, 262144, 300001])
def test_offsets_bit_exact(rec, n):
    lengths = rng.integers(0, 101, size=n).astype(np.int32)
    got = rec.sls_offsets(dev(lengths)).cpu().numpy()
    assert np.array_equal(got, oracle.offsets(lengths))


def test_offsets_need_64_bits(rec):
    lengths = np.full(5000, 2**31 - 1, np.int32)
    got = rec.sls_offsets(dev(lengths)).cpu().numpy()
    assert np.array_equal(got, oracle.offsets(lengths))


def test_split_query_matches_oracle(rec):
    for n in [0, 1, 15, 16, 17, 145, 999, 1000]:
        for B in synth.SWEEP_BATCH_SIZES:
            assert rec.split_query(n, B) == oracle.split_query(n, B)


def test_validate_matches_oracle(rec):
    T, B, R = 5, 300, 1000
    rows = [R, R // 2, R, 7, R]
    lengths = rng.integers(0, 90, size=T * B).astype(np.int32)
    off = oracle.offsets(lengths)
    idx = np.concatenate([rng.integers(0, rows[t], size=int(off[(t + 1) * B] - off[t * B])) for t in range(T)]).astype(np.int32)
    assert rec.sls_validate(rows, dev(idx), dev(lengths), B) == oracle.validate(rows, idx, lengths, B) == (rec.OK, 0, -1)
    bad = idx.copy()
    pos = rng.choice(idx.size, size=37, replace=False)
    bad[pos] = rng.choice([-1, -2**31, 2**31 - 1, R], size=37)
    # also an index that is legal for table 0 but not for the 7-row table 3
    p3 = int(off[3 * B]) + 5
    bad[p3] = 7
    want = oracle.validate(rows, bad, lengths, B)
    assert want[0] == oracle.ERR_INDEX_RANGE
    assert rec.sls_validate(rows, dev(bad), dev(lengths), B) == want
    neg = lengths.copy(); neg[77] = -3
    assert rec.sls_validate(rows, dev(idx), dev(neg), B)[0] == oracle.validate(rows, idx, neg, B)[0] == rec.ERR_NEGATIVE_LENGTH
    assert rec.sls_validate(rows, dev(idx[:-1]), dev(lengths), B)[0] == oracle.validate(rows, idx[:-1], lengths, B)[0] \
        == rec.ERR_LENGTHS_MISMATCH
    # all-empty bags
    z = np.zeros(T * B, np.int32)
    assert rec.sls_validate(rows, dev(np.zeros(0, np.int32)), dev(z), B) == (rec.OK, 0, -1)


def test_bf16_conversion_bit_exact(rec):
    x = np.concatenate([rng.normal(size=100_000) * 10.0 ** rng.integers(-8, 8, size=100_000),
                        np.array([0.0, -0.0, 1.0, 1 + 2.0**-8, 1 + 3 * 2.0**-8, np.inf, -np.inf, 3.4e38, 1e-40, np.nan])]
                       ).astype(np.float32)
    got = rec.f32_to_bf16(dev(x)).cpu().numpy().view(np.uint16)
    want = (oracle.bf16_round(x).view(np.uint32) >> 16).astype(np.uint16)
    assert np.array_equal(got, want)


# ------------------------------------------------------------------ SLS

@pytest.mark.parametrize("D", [4, 16, 32, 48, 64, 128, 256])
def test_sls_ragged_vs_oracle(rec, D):
    T, B, R = 3, 37, 500
    tables = [rng.uniform(-0.05, 0.05, size=(R, D)).astype(np.float32) for _ in range(T)]
    idx, lengths = _bags(T, B, R, 0, 150)
    lengths[5] = 0
    idx, lengths = idx[: int(lengths.sum())], lengths
    idx = rng.integers(0, R, size=int(lengths.sum())).astype(np.int32)
    E, _, aabs = oracle.sls(tables, idx, lengths, B, extra=True)
    got = rec.sls_forward(rec.Tables([dev(t) for t in tables]), dev(idx), dev(lengths), B).cpu().numpy()
    assert_close(got, E, TOL_F32, f"SLS D={D}")
    # summation-error bound for any order of L fp32 adds
    L = lengths.reshape(T, B).T[:, :, None]
    assert np.all(np.abs(got.astype(np.float64) - E) <= (L + 1) * 2.0**-24 * aabs + 1e-30)


@pytest.mark.parametrize("D", [4, 16, 32, 48, 64, 128, 256])
def test_sls_short_bags_vs_oracle(rec, D):
    """Average bag length <= 2 takes the kernel that pools several bags per wavefront; one long
    bag among them must still come out right."""
    T, B, R = 3, 400, 300
    tables = [rng.uniform(-0.05, 0.05, size=(R, D)).astype(np.float32) for _ in range(T)]
    lengths = rng.integers(0, 4, size=T * B).astype(np.int32)
    lengths[7] = 200
    lengths[T * B - 1] = 3
    assert lengths.sum() <= 2 * T * B
    idx = rng.integers(0, R, size=int(lengths.sum())).astype(np.int32)
    E, _, aabs = oracle.sls(tables, idx, lengths, B, extra=True)
    got = rec.sls_forward(rec.Tables([dev(t) for t in tables]), dev(idx), dev(lengths), B).cpu().numpy()
    assert_close(got, E, TOL_F32, f"short-bag SLS D={D}")
    L = lengths.reshape(T, B).T[:, :, None]
    assert np.all(np.abs(got.astype(np.float64) - E) <= (L + 1) * 2.0**-24 * aabs + 1e-30)
    # one lookup per bag is a gather, exactly
    idx1 = rng.integers(0, R, size=T * B).astype(np.int32)
    got1 = rec.sls_forward(rec.Tables([dev(t) for t in tables]), dev(idx1), dev(np.ones(T * B, np.int32)), B).cpu().numpy()
    for t in range(T):
        assert np.array_equal(got1[:, t, :], tables[t][idx1[t * B:(t + 1) * B]])


def test_sls_integer_tables_exact_and_special_lengths(rec):
    T, B, R, D = 4, 50, 64, 32
    tables = [rng.integers(-8, 9, size=(R, D)).astype(np.float32) for _ in range(T)]
    tabs = rec.Tables([dev(t) for t in tables])
    for lo, hi in [(0, 0), (1, 1), (0, 3), (63, 65), (127, 130), (1000, 1000)]:
        idx, lengths = _bags(T, B, R, lo, hi)
        got = rec.sls_forward(tabs, dev(idx), dev(lengths), B).cpu().numpy()
        assert np.array_equal(got, oracle.sls(tables, idx, lengths, B)), (lo, hi)
    # all-ones lengths: a pure gather
    idx = rng.integers(0, R, size=T * B).astype(np.int32)
    got = rec.sls_forward(tabs, dev(idx), dev(np.ones(T * B, np.int32)), B).cpu().numpy()
    for t in range(T):
        assert np.array_equal(got[:, t, :], tables[t][idx[t * B:(t + 1) * B]])


def test_sls_strided_output_and_different_table_sizes(rec):
    D, B = 64, 19
    rows = [10, 1000, 3]
    tables = [rng.uniform(-1, 1, size=(r, D)).astype(np.float32) for r in rows]
    T, V = 3, 4
    lengths = rng.integers(0, 40, size=T * B).astype(np.int32)
    off = oracle.offsets(lengths)
    idx = np.concatenate([rng.integers(0, rows[t], size=int(off[(t + 1) * B] - off[t * B])) for t in range(T)]).astype(np.int32)
    buf = torch.full((B, V, D), -7.0, dtype=torch.float32, device="cuda")
    rec.sls_forward(rec.Tables([dev(t) for t in tables]), dev(idx), dev(lengths), B, out=buf[:, 1:, :],
                    out_stride_b=V * D, out_stride_t=D)
    got = buf.cpu().numpy()
    assert np.all(got[:, 0, :] == -7.0)                 # slot 0 untouched
    assert_close(got[:, 1:, :], oracle.sls(tables, idx, lengths, B), TOL_F32, "strided SLS")


def test_sls_is_deterministic(rec):
    cfg = synth.CONFIGS["tiny"]
    tabs = rec.Tables([dev(synth.table_full(cfg, t)) for t in range(cfg.T)])
    b = synth.BatchGenerator(cfg).batch(0)
    a1 = rec.sls_forward(tabs, dev(b.indices), dev(b.lengths), cfg.B)
    a2 = rec.sls_forward(tabs, dev(b.indices), dev(b.lengths), cfg.B)
    assert torch.equal(a1, a2)


# ------------------------------------------------------------------ interaction

@pytest.mark.parametrize("V,D,B", [(2, 4, 3), (9, 32, 64), (11, 32, 100), (41, 64, 33), (27, 128, 5), (33, 12, 7),
                                   (65, 64, 9), (128, 100, 3), (100, 256, 2), (32, 8, 1025)])
def test_interact_vs_oracle(rec, V, D, B):
    v = rng.normal(size=(B, V, D)).astype(np.float32)
    got = rec.interact(dev(v)).cpu().numpy()
    want = oracle.interact(v)
    assert np.array_equal(got[:, :D], v[:, 0, :])          # the copy is exact
    assert_close(got, want, TOL_F32, f"interact V={V} D={D}")
    vi = rng.integers(-4, 5, size=(B, V, D)).astype(np.float32)
    assert np.array_equal(rec.interact(dev(vi)).cpu().numpy(), oracle.interact(vi))


# ------------------------------------------------------------------ FC stacks

@pytest.mark.parametrize("widths,B", [((13, 64, 32), 64), ((13, 256, 128, 64), 100), ((87, 256, 64, 1), 257),
                                      ((884, 512, 128, 1), 1024), ((5, 1), 1), ((70, 33, 65, 2), 63),
                                      ((20, 24, 28, 32, 36, 40, 3), 50), ((64, 32, 1000, 16), 40),
                                      ((512, 512, 7), 17), ((600, 64, 700, 5), 33),
                                      ((320, 8), 33), ((448, 40, 17), 20), ((192, 100), 16), ((384, 24), 5),
                                      ((896, 512), 1024), ((512, 700), 900), ((256, 1024, 8), 1500), ((288, 130), 2100),
                                      ((256, 16424), 3), ((512, 12800, 5), 1)])
def test_mlp_f32_vs_oracle(rec, widths, B):
    p = synth.mlp_params(widths, stack=3)
    x = rng.uniform(0, 1, size=(B, widths[0])).astype(np.float32)
    W, b = [dev(w) for w in p.W], [dev(v) for v in p.b]
    for hidden, final in [(rec.ACT_RELU, rec.ACT_RELU), (rec.ACT_RELU, rec.ACT_SIGMOID), (rec.ACT_NONE, rec.ACT_NONE)]:
        got = rec.mlp_forward(W, b, dev(x), hidden, final).cpu().numpy()
        want = oracle.mlp(x, p.W, p.b, hidden, final)
        assert_close(got, want, TOL_F32, f"fp32 MLP {widths} acts {hidden},{final}")


def test_mlp_f32_exact_cases(rec):
    xi = rng.integers(-4, 5, size=(70, 40)).astype(np.float32)
    Wi = rng.integers(-4, 5, size=(33, 40)).astype(np.float32)
    bi = rng.integers(-4, 5, size=33).astype(np.float32)
    got = rec.mlp_forward([dev(Wi)], [dev(bi)], dev(xi), final_act=rec.ACT_NONE).cpu().numpy()
    assert np.array_equal(got, xi @ Wi.T + bi)
    got = rec.mlp_forward([dev(np.zeros((1, 40), np.float32))], [dev(np.zeros(1, np.float32))], dev(xi),
                          final_act=rec.ACT_SIGMOID).cpu().numpy()
    assert np.array_equal(got, np.full((70, 1), 0.5, np.float32))


@pytest.mark.parametrize("widths,B", [((2560, 1024, 256, 32), 128), ((87, 512, 256, 1), 300), ((64, 8), 5),
                                      ((100, 70, 3), 65), ((20, 24, 28, 32, 36, 40, 3), 50),
                                      ((64, 32, 1100, 16), 40), ((1024, 128, 9), 17),
                                      ((512, 700), 600), ((512, 1024, 640, 8), 900), ((2560, 1024), 1024),
                                      ((640, 8), 33), ((1024, 40, 17), 20), ((896, 100), 16),
                                      ((256, 16424), 3), ((256, 8200, 9), 1), ((320, 16424), 70)])
def test_mlp_bf16_vs_oracle(rec, widths, B):
    oracle.set_threads(16)
    p = synth.mlp_params(widths, stack=4)
    x = rng.normal(size=(B, widths[0])).astype(np.float32)
    W, b = [rec.f32_to_bf16(dev(w)) for w in p.W], [dev(v) for v in p.b]
    final = rec.ACT_SIGMOID if widths[-1] == 1 else rec.ACT_RELU
    got = rec.mlp_forward(W, b, dev(x), rec.ACT_RELU, final, wdtype=rec.BF16).cpu().numpy()
    want = oracle.mlp(x, p.W, p.b, rec.ACT_RELU, final, bf16=True)
    assert_close(got, want, TOL_BF16, f"bf16 MLP {widths}")
    if widths[0] >= 64 and len(widths) > 2:
        # operands really are bf16: the result is measurably away from the unrounded one
        full = oracle.mlp(x, p.W, p.b, rec.ACT_RELU, final)
        assert rel_err(got, full) > 1e-4


def test_mlp_bf16_exact_on_small_integers(rec):
    xi = rng.integers(-4, 5, size=(70, 48)).astype(np.float32)
    Wi = rng.integers(-4, 5, size=(33, 48)).astype(np.float32)
    bi = rng.integers(-4, 5, size=33).astype(np.float32)
    got = rec.mlp_forward([rec.f32_to_bf16(dev(Wi))], [dev(bi)], dev(xi), final_act=rec.ACT_NONE, wdtype=rec.BF16)
    assert np.array_equal(got.cpu().numpy(), xi @ Wi.T + bi)


# ------------------------------------------------------------------ whole model, reduced sizes

def _host_model(cfg):
    return [synth.table_full(cfg, t) for t in range(cfg.T)]


@pytest.mark.parametrize("name,R,B", [("tiny", 10_000, 64), ("rmc1", 3000, 70), ("rmc2", 2000, 45), ("rmc3", 3000, 130)])
def test_model_forward_small(rec, name, R, B):
    from paper_2001_02772_amd import workload
    cfg = synth.CONFIGS[name].replace(R=R, B=B)
    tables = _host_model(cfg)
    model = workload.device_model(cfg, tables=rec.Tables([dev(t) for t in tables]))
    batch = synth.BatchGenerator(cfg).batch(2)
    db = workload.DeviceBatch(batch)
    assert rec.sls_validate([R] * cfg.T, db.indices, db.lengths, B) == (rec.OK, 0, -1)
    got = model.forward(db.dense, db.indices, db.lengths, B).cpu().numpy()
    want = oracle_forward(cfg, tables, batch)
    assert np.all((got > 0) & (got < 1))
    assert_close(got, want, TOL_BF16 if cfg.bf16 else TOL_F32, f"model {name}")
    # query splitting: any partition into sub-batches gives the same per-sample outputs
    parts = rec.split_query(B, 16)
    pieces = []
    for start, count in parts:
        sb = workload.DeviceBatch(workload.slice_batch(batch, cfg.T, start, count))
        pieces.append(model.forward(sb.dense, sb.indices, sb.lengths, count).cpu().numpy())
    assert_close(np.concatenate(pieces), want, TOL_BF16 if cfg.bf16 else TOL_F32, f"split model {name}")
    # deterministic
    assert np.array_equal(got, model.forward(db.dense, db.indices, db.lengths, B).cpu().numpy())
    # host-only create: the padded copy of the first predictor layer in a caller-provided buffer, filled by
    # rec_model_prepare, gives the same bits as the copy rec_model_create allocates itself
    other = workload.device_model(cfg, tables=model.tables, caller_padded_weights=True)
    assert (other._padded is not None) == (model.padded_weight_bytes > 0)
    assert np.array_equal(got, other.forward(db.dense, db.indices, db.lengths, B).cpu().numpy())


CONCAT_VARIANTS = {
    "wnd-tiny": synth.CONFIGS["wnd-tiny"],
    "wnd-small-bf16": synth.CONFIGS["wnd"].replace(R=3000, B=70),
    "wnd-tiny-bf16": synth.CONFIGS["wnd-tiny"].replace(bf16=True),
    # a dense stack in front of the join, several lookups per bag (pooled sums are joined)
    "concat-with-dense-stack": synth.CONFIGS["wnd-tiny"].replace(bottom=(16, 24, 12), top=(12 + 5 * 8, 32, 1), len_lo=0,
                                                                 len_hi=6, B=37),
    # wide join: the first predictor layer takes the tiled kernel's split-k path
    "concat-wide": synth.CONFIGS["wnd-tiny"].replace(F=256, bottom=(256,), T=12, D=64, top=(256 + 12 * 64, 128, 1), B=200),
}


@pytest.mark.parametrize("name", sorted(CONCAT_VARIANTS))
def test_concat_model_forward_small(rec, name):
    from paper_2001_02772_amd import workload
    cfg = CONCAT_VARIANTS[name]
    synth.check_config(cfg)
    tables = _host_model(cfg)
    model = workload.device_model(cfg, tables=rec.Tables([dev(t) for t in tables]))
    batch = synth.BatchGenerator(cfg).batch(3)
    db = workload.DeviceBatch(batch)
    got = model.forward(db.dense, db.indices, db.lengths, cfg.B).cpu().numpy()
    want = oracle_forward(cfg, tables, batch)
    assert np.all((got >= 0) & (got <= 1))
    assert_close(got, want, TOL_BF16 if cfg.bf16 else TOL_F32, f"concat model {name}")
    pieces = []
    for start, count in rec.split_query(cfg.B, 16):
        sb = workload.DeviceBatch(workload.slice_batch(batch, cfg.T, start, count))
        pieces.append(model.forward(sb.dense, sb.indices, sb.lengths, count).cpu().numpy())
    assert_close(np.concatenate(pieces), want, TOL_BF16 if cfg.bf16 else TOL_F32, f"split concat model {name}")


def test_concat_model_create_errors(rec):
    cfg = synth.CONFIGS["wnd-tiny"]
    tables = rec.Tables([dev(t) for t in _host_model(cfg)])
    from paper_2001_02772_amd import workload
    Wt, bt = workload.device_mlp(synth.mlp_params((57, 8, 1), 1), False)
    with pytest.raises(rec.RecError) as e:                         # predictor input != F + T*D
        rec.Model(tables, [], [], Wt, bt, interaction=rec.INTERACT_CONCAT, dense_features=16)
    assert e.value.status == rec.ERR_BAD_SHAPE
    Wt, bt = workload.device_mlp(synth.mlp_params((55, 8, 1), 1), False)
    with pytest.raises(rec.RecError) as e:                         # joined dense part not a multiple of 4 wide
        rec.Model(tables, [], [], Wt, bt, interaction=rec.INTERACT_CONCAT, dense_features=15)
    assert e.value.status == rec.ERR_UNSUPPORTED
    with pytest.raises(rec.RecError) as e:                         # the dot interaction needs a dense stack
        rec.Model(tables, [], [], Wt, bt, interaction=rec.INTERACT_DOT, dense_features=16)
    assert e.value.status == rec.ERR_BAD_SHAPE


@pytest.mark.parametrize("name,B", [("tiny", 5000), ("tiny", 40000), ("wnd-tiny", 3000)])
def test_model_forward_large_batch(rec, name, B):
    """Batches far above the benchmark's: T*B = 320,000 bags is past the scan's parallel tiles, so the
    scan runs as one block with a carry and gets a launch of its own instead of riding with the
    dense stack."""
    from paper_2001_02772_amd import workload
    import oracle as orc
    cfg = synth.CONFIGS[name].replace(B=B)
    tables = _host_model(cfg)
    model = workload.device_model(cfg, tables=rec.Tables([dev(t) for t in tables]))
    batch = synth.BatchGenerator(cfg).batch(5)
    db = workload.DeviceBatch(batch)
    got = model.forward(db.dense, db.indices, db.lengths, B).cpu().numpy()
    orc.set_threads(16)
    want = oracle_forward(cfg, tables, batch)
    orc.set_threads(1)
    assert_close(got, want, TOL_F32, f"large-batch model {name} B={B}")


def test_model_edge_cases(rec):
    from paper_2001_02772_amd import workload
    cfg = synth.CONFIGS["tiny"].replace(R=100)
    tables = _host_model(cfg)
    model = workload.device_model(cfg, tables=rec.Tables([dev(t) for t in tables]))
    # B = 0: nothing to do
    e = torch.zeros(0, device="cuda")
    assert model.forward(e, e.int(), e.int(), 0).numel() == 0
    # B = 1 with all bags empty, and one very long bag
    for lens in [np.zeros(cfg.T, np.int32), np.array([1000] + [0] * (cfg.T - 1), np.int32)]:
        idx = rng.integers(0, 100, size=int(lens.sum())).astype(np.int32)
        b = synth.Batch(1, rng.uniform(size=(1, cfg.F)).astype(np.float32), lens, idx)
        db = workload.DeviceBatch(b)
        got = model.forward(db.dense, db.indices, db.lengths, 1).cpu().numpy()
        assert_close(got, oracle_forward(cfg, tables, b), TOL_F32, "edge")


def test_host_checkable_errors(rec):
    t = rec.Tables([dev(np.zeros((4, 8), np.float32))])
    idx, lens = dev(np.zeros(2, np.int32)), dev(np.ones(2, np.int32))
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(rec.RecError) as e:
        rec.sls_forward(t, idx, lens, 2, workspace=small[:16])
    assert e.value.status == rec.ERR_WORKSPACE
    bad = rec.Tables([dev(np.zeros((4, 6), np.float32))])      # D not a multiple of 4
    with pytest.raises(rec.RecError) as e:
        rec.sls_forward(bad, idx, lens, 2)
    assert e.value.status == rec.ERR_UNSUPPORTED
    with pytest.raises(rec.RecError) as e:
        rec.interact(dev(np.zeros((2, 3, 8), np.float32)), out=torch.empty((2, 4), device="cuda"), ldo=4)
    assert e.value.status == rec.ERR_BAD_SHAPE
    assert rec.status_string(rec.ERR_INDEX_RANGE) == "REC_ERR_INDEX_RANGE"


@pytest.mark.parametrize("widths,B", [((2560, 1024), 2048), ((2560, 1024), 4000), ((2560, 1024), 16300),
                                      ((256, 4136), 3300), ((2560, 1024, 8), 4000), ((1024, 512, 1), 5000)])
def test_mlp_bf16_large_batches_sampled_rows(rec, widths, B):
    """Batches that put the wide layer on the larger tile shapes (128x64, 128x128, 256x256, ragged in
    both directions).  The oracle computes a sample of the rows -- rows are independent -- taken from
    the first tile, the ragged last tile and in between."""
    oracle.set_threads(16)
    p = synth.mlp_params(widths, stack=5)
    g = np.random.default_rng(B)
    x = g.normal(size=(B, widths[0])).astype(np.float32)
    rows = np.unique(np.concatenate([np.arange(40), np.arange(B - 70, B), g.integers(0, B, size=150)]))
    W, b = [rec.f32_to_bf16(dev(w)) for w in p.W], [dev(v) for v in p.b]
    final = rec.ACT_SIGMOID if widths[-1] == 1 else rec.ACT_RELU
    got = rec.mlp_forward(W, b, dev(x), rec.ACT_RELU, final, wdtype=rec.BF16).cpu().numpy()
    want = oracle.mlp(x[rows], p.W, p.b, rec.ACT_RELU, final, bf16=True)
    assert got.shape == (B, widths[-1])
    assert_close(got[rows], want, TOL_BF16, f"bf16 MLP {widths} at B={B}, {rows.size} sampled rows")
    assert np.isfinite(got).all()
