"""Pins for the CPU oracle: each oracle function is checked against something
other than itself -- hand-worked fixtures, closed forms, invariants, and NumPy /
PyTorch-CPU library routines.  CPU only."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2001_02772_amd import synth

rng = np.random.default_rng(7)


def _tables(T, R, D, integer=False):
    if integer:
        return [rng.integers(-8, 9, size=(R, D)).astype(np.float32) for _ in range(T)]
    return [rng.uniform(-0.05, 0.05, size=(R, D)).astype(np.float32) for _ in range(T)]


def _bags(T, B, R, lo, hi):
    lengths = rng.integers(lo, hi + 1, size=T * B).astype(np.int32)
    indices = rng.integers(0, R, size=int(lengths.sum())).astype(np.int32)
    return indices, lengths


# ---------------------------------------------------------------- validator

def test_validate_ok_and_each_error():
    rows = [5, 3]
    lengths = np.array([3, 0, 4, 1, 2, 3], np.int32)
    idx = np.array([0, 2, 2, 4, 1, 3, 0, 1, 2, 0, 2, 2, 2], np.int32)
    assert oracle.validate(rows, idx, lengths, 3) == (oracle.OK, 0, -1)
    bad = lengths.copy(); bad[1] = -1
    assert oracle.validate(rows, idx, bad, 3)[0] == oracle.ERR_NEGATIVE_LENGTH
    assert oracle.validate(rows, idx[:-1], lengths, 3)[0] == oracle.ERR_LENGTHS_MISMATCH
    assert oracle.validate(rows, np.append(idx, 0), lengths, 3)[0] == oracle.ERR_LENGTHS_MISMATCH
    # index 3 is fine for table 0 (5 rows) but out of range for table 1 (3 rows)
    j = idx.copy(); j[8] = 3; j[12] = -1
    assert oracle.validate(rows, j, lengths, 3) == (oracle.ERR_INDEX_RANGE, 2, 8)
    j = idx.copy(); j[3] = 5
    assert oracle.validate(rows, j, lengths, 3) == (oracle.ERR_INDEX_RANGE, 1, 3)
    # boundary: rows-1 is legal
    j = idx.copy(); j[0] = 4; j[7] = 2
    assert oracle.validate(rows, j, lengths, 3) == (oracle.OK, 0, -1)


def test_validate_brute_force_counts():
    T, B, R = 3, 17, 11
    idx, lengths = _bags(T, B, R, 0, 6)
    idx = idx.copy()
    pos = rng.choice(idx.size, size=9, replace=False)
    idx[pos] = rng.choice([-1, -7, R, R + 5], size=9)
    st, n_bad, first = oracle.validate([R] * T, idx, lengths, B)
    assert (st, n_bad, first) == (oracle.ERR_INDEX_RANGE, 9, int(pos.min()))


def test_validate_per_table_row_counts():
    rows = [4, 100]
    lengths = np.array([1, 1, 1, 1], np.int32)       # T=2, B=2
    assert oracle.validate(rows, [3, 3, 99, 50], lengths, 2)[0] == oracle.OK
    assert oracle.validate(rows, [3, 50, 99, 50], lengths, 2) == (oracle.ERR_INDEX_RANGE, 1, 1)


def test_validate_empty():
    assert oracle.validate([5], np.zeros(0, np.int32), np.zeros(0, np.int32), 0) == (oracle.OK, 0, -1)
    assert oracle.validate([5], np.zeros(0, np.int32), np.zeros(4, np.int32), 4) == (oracle.OK, 0, -1)


# ---------------------------------------------------------------- offsets / split

def test_offsets_closed_form_and_cumsum():
    assert oracle.offsets(np.full(50, 7, np.int32)).tolist() == [7 * i for i in range(51)]
    L = rng.integers(0, 100, size=1000).astype(np.int32)
    assert np.array_equal(oracle.offsets(L)[1:], np.cumsum(L, dtype=np.int64))
    assert oracle.offsets(np.zeros(0, np.int32)).tolist() == [0]
    # needs 64 bits
    big = np.full(3, 2**31 - 1, np.int32)
    assert oracle.offsets(big).tolist() == [0, 2**31 - 1, 2 * (2**31 - 1), 3 * (2**31 - 1)]


def test_split_query_closed_forms():
    assert oracle.split_query(10, 4) == [(0, 4), (4, 4), (8, 2)]
    assert oracle.split_query(8, 4) == [(0, 4), (4, 4)]
    assert oracle.split_query(3, 1024) == [(0, 3)]
    assert oracle.split_query(0, 16) == []
    for n in range(1, 200):
        for B in (1, 7, 16, 64, 256):
            s = oracle.split_query(n, B)
            assert len(s) == math.ceil(n / B)
            assert sum(c for _, c in s) == n
            assert all(c == B for _, c in s[:-1]) and 1 <= s[-1][1] <= B
            assert [a for a, _ in s] == [i * B for i in range(len(s))]


# ---------------------------------------------------------------- SLS

def test_sls_hand_computed(golden):
    g = golden("sls_hand_bags.txt")
    D, B = int(g["D"][0]), int(g["B"][0])
    tables = [np.array(g["table0"], np.float32).reshape(-1, D), np.array(g["table1"], np.float32).reshape(-1, D)]
    lengths, idx = np.array(g["lengths"], np.int32), np.array(g["indices"], np.int32)
    assert oracle.offsets(lengths).tolist() == [int(v) for v in g["offsets"]]
    E, seq, aabs = oracle.sls(tables, idx, lengths, B, extra=True)
    for b in range(B):
        for t in range(2):
            want = np.array(g[f"E_b{b}_t{t}"], np.float32)
            assert np.array_equal(E[b, t], want), (b, t)
            assert np.array_equal(seq[b, t], want), (b, t)
    # sum of |x| for bag (t0,b0): |r0| + 2|r2|
    assert aabs[0, 0].tolist() == [21.0, 8.0, 3.0, 6.0]


def test_sls_all_ones_is_gather_and_zero_lengths_give_zero():
    T, B, R, D = 3, 9, 50, 16
    tables = _tables(T, R, D)
    idx = rng.integers(0, R, size=T * B).astype(np.int32)
    E = oracle.sls(tables, idx, np.ones(T * B, np.int32), B)
    for t in range(T):
        assert np.array_equal(E[:, t, :], tables[t][idx[t * B:(t + 1) * B]])
    Z = oracle.sls(tables, np.zeros(0, np.int32), np.zeros(T * B, np.int32), B)
    assert not Z.any() and not np.signbit(Z).any()


def test_sls_equals_count_matrix_product():
    """The lookup-and-pool equals a sparse (multiplicity) matrix times the table
    (Section II-A, last sentence of "Embedding Table Access")."""
    T, B, R, D = 4, 13, 37, 8
    tables = _tables(T, R, D)
    idx, lengths = _bags(T, B, R, 0, 30)
    E = oracle.sls(tables, idx, lengths, B)
    off = np.concatenate([[0], np.cumsum(lengths)])
    for t in range(T):
        S = np.zeros((B, R), dtype=np.float64)
        for b in range(B):
            for p in range(off[t * B + b], off[t * B + b + 1]):
                S[b, idx[p]] += 1.0
        want = (S @ tables[t].astype(np.float64)).astype(np.float32)
        # both are fp64 sums of <=30 fp32 terms: they can differ by one final rounding at most
        assert np.allclose(E[:, t, :], want, rtol=0, atol=2e-9)


def test_sls_matches_torch_embedding_bag():
    T, B, R, D = 2, 21, 101, 32
    tables = _tables(T, R, D)
    idx, lengths = _bags(T, B, R, 0, 100)
    E, seq, aabs = oracle.sls(tables, idx, lengths, B, extra=True)
    off = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    for t in range(T):
        lo, hi = off[t * B], off[(t + 1) * B]
        want = torch.nn.functional.embedding_bag(
            torch.from_numpy(idx[lo:hi].astype(np.int64)), torch.from_numpy(tables[t]).double(),
            torch.from_numpy(off[t * B:(t + 1) * B] - lo), mode="sum").numpy()
        assert np.array_equal(E[:, t, :], want.astype(np.float32))
        # the fp32 in-order sum obeys the textbook bound (L-1) u sum|x| (first order)
        L = lengths[t * B:(t + 1) * B][:, None]
        assert np.all(np.abs(seq[:, t, :].astype(np.float64) - want) <= (L + 1) * 2.0**-24 * aabs[:, t, :] + 1e-30)


def test_sls_permutation_concatenation_linearity():
    T, B, R, D = 2, 6, 40, 8
    tab_i = _tables(T, R, D, integer=True)
    idx, lengths = _bags(T, B, R, 1, 25)
    E = oracle.sls(tab_i, idx, lengths, B)
    # permuting lookups inside each bag: exact with integer-valued rows
    off = np.concatenate([[0], np.cumsum(lengths)])
    perm_idx = idx.copy()
    for i in range(T * B):
        perm_idx[off[i]:off[i + 1]] = rng.permutation(idx[off[i]:off[i + 1]])
    assert np.array_equal(oracle.sls(tab_i, perm_idx, lengths, B), E)
    # scaling a table by two doubles the result bit-exactly (any values)
    tab_f = _tables(T, R, D)
    Ef = oracle.sls(tab_f, idx, lengths, B)
    assert np.array_equal(oracle.sls([2 * t for t in tab_f], idx, lengths, B), 2 * Ef)
    # bag concatenation: SLS(bag1 ‖ bag2) = SLS(bag1) + SLS(bag2)   (integer rows: exact)
    idx2, len2 = _bags(T, B, R, 0, 10)
    off2 = np.concatenate([[0], np.cumsum(len2)])
    cat = np.concatenate([np.concatenate([idx[off[i]:off[i + 1]], idx2[off2[i]:off2[i + 1]]]) for i in range(T * B)])
    assert np.array_equal(oracle.sls(tab_i, cat.astype(np.int32), lengths + len2, B),
                          E + oracle.sls(tab_i, idx2, len2, B))


def test_sls_bag_order_is_table_major():
    # table 0 holds 1s, table 1 holds 100s; lengths differ per (t, b)
    tables = [np.ones((4, 2), np.float32), np.full((4, 2), 100, np.float32)]
    lengths = np.array([1, 2, 3, 4, 5, 6], np.int32)      # (t0,b0..b2), (t1,b0..b2)
    idx = np.zeros(21, np.int32)
    E = oracle.sls(tables, idx, lengths, 3)
    assert E[:, 0, 0].tolist() == [1, 2, 3] and E[:, 1, 0].tolist() == [400, 500, 600]


# ---------------------------------------------------------------- FC

def test_fc_vs_numpy_float64_non_square():
    B, n_in, n_out = 19, 37, 11
    x = rng.normal(size=(B, n_in)).astype(np.float32)
    W = rng.normal(size=(n_out, n_in)).astype(np.float32)
    b = rng.normal(size=n_out).astype(np.float32)
    z = x.astype(np.float64) @ W.astype(np.float64).T + b.astype(np.float64)
    assert np.allclose(oracle.fc(x, W, b, oracle.ACT_NONE), z, rtol=1e-7, atol=1e-7)
    assert np.allclose(oracle.fc(x, W, b, oracle.ACT_RELU), np.maximum(z, 0), rtol=1e-7, atol=1e-7)
    assert np.allclose(oracle.fc(x, W, b, oracle.ACT_SIGMOID), 1 / (1 + np.exp(-z)), rtol=1e-7, atol=0)
    want = torch.nn.functional.linear(torch.from_numpy(x).double(), torch.from_numpy(W).double(),
                                      torch.from_numpy(b).double()).numpy()
    assert np.allclose(oracle.fc(x, W, b, oracle.ACT_NONE), want, rtol=1e-7, atol=1e-7)


def test_fc_special_cases():
    x = rng.normal(size=(5, 6)).astype(np.float32)
    I, zb = np.eye(6, dtype=np.float32), np.zeros(6, np.float32)
    assert np.array_equal(oracle.fc(x, I, zb, oracle.ACT_RELU), np.maximum(x, 0))
    assert np.array_equal(oracle.fc(x, I, zb, oracle.ACT_NONE), x)
    b = rng.normal(size=6).astype(np.float32)
    assert np.array_equal(oracle.fc(x, np.zeros((6, 6), np.float32), b, oracle.ACT_NONE), np.tile(b, (5, 1)))
    # zero last layer -> probability exactly one half
    assert np.array_equal(oracle.fc(x, np.zeros((1, 6), np.float32), np.zeros(1, np.float32), oracle.ACT_SIGMOID),
                          np.full((5, 1), 0.5, np.float32))
    # integer-valued inputs: exact
    xi = rng.integers(-4, 5, size=(3, 8)).astype(np.float32)
    Wi = rng.integers(-4, 5, size=(2, 8)).astype(np.float32)
    assert np.array_equal(oracle.fc(xi, Wi, np.zeros(2, np.float32), oracle.ACT_NONE), xi @ Wi.T)
    assert np.array_equal(oracle.fc(xi, Wi, np.zeros(2, np.float32), oracle.ACT_NONE, bf16=True), xi @ Wi.T)


def test_bf16_round_vs_torch_and_cases():
    x = np.concatenate([rng.normal(size=4096).astype(np.float32) * 10.0 ** rng.integers(-6, 6, size=4096),
                        np.array([0.0, -0.0, 1.0, np.inf, -np.inf, 3.4e38, 1e-40], np.float32)])
    want = torch.from_numpy(x).to(torch.bfloat16).float().numpy()
    got = oracle.bf16_round(x)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    # ties to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7 -> 1 ; 1 + 3*2^-8 -> 1 + 2^-6
    assert oracle.bf16_round(np.float32([1 + 2.0**-8]))[0] == 1.0
    assert oracle.bf16_round(np.float32([1 + 3 * 2.0**-8]))[0] == np.float32(1 + 2.0**-6)
    assert np.isnan(oracle.bf16_round(np.float32([np.nan]))[0])


def test_fc_bf16_operand_rounding():
    B, n_in, n_out = 7, 300, 5
    x = rng.normal(size=(B, n_in)).astype(np.float32)
    W = (rng.normal(size=(n_out, n_in)) / 17).astype(np.float32)
    b = rng.normal(size=n_out).astype(np.float32)
    xr = torch.from_numpy(x).to(torch.bfloat16).double().numpy()
    Wr = torch.from_numpy(W).to(torch.bfloat16).double().numpy()
    want = xr @ Wr.T + b
    got = oracle.fc(x, W, b, oracle.ACT_NONE, bf16=True)
    assert np.allclose(got, want, rtol=1e-7, atol=1e-7)
    # and it really differs from the unrounded product at the 2^-9 scale
    full = oracle.fc(x, W, b, oracle.ACT_NONE)
    rel = np.abs(got - full).max() / np.abs(full).max()
    assert 1e-5 < rel < 2e-2


def test_mlp_is_composition_of_layers():
    widths = (13, 20, 9, 1)
    p = synth.mlp_params(widths, stack=0)
    x = rng.uniform(size=(11, 13)).astype(np.float32)
    h = x.astype(np.float64)
    for l in range(3):
        h = h @ p.W[l].astype(np.float64).T + p.b[l]
        h = np.maximum(h, 0) if l < 2 else 1 / (1 + np.exp(-h))
        h = h.astype(np.float32).astype(np.float64)
    got = oracle.mlp(x, p.W, p.b, oracle.ACT_RELU, oracle.ACT_SIGMOID)
    assert np.allclose(got, h, rtol=2e-7, atol=0)


# ---------------------------------------------------------------- interaction

def test_interact_hand_example(golden):
    g = golden("interact_hand_example.txt")
    out = oracle.interact(np.array(g["vecs"], np.float32).reshape(1, 3, 2))
    assert out[0].tolist() == g["out"]


def test_interact_vs_einsum_tril_order():
    B, V, D = 5, 9, 16
    v = rng.normal(size=(B, V, D)).astype(np.float32)
    out = oracle.interact(v)
    Z = np.einsum("bid,bjd->bij", v.astype(np.float64), v.astype(np.float64))
    assert np.allclose(Z, Z.transpose(0, 2, 1))
    i, j = np.tril_indices(V, -1)
    assert out.shape == (B, D + V * (V - 1) // 2)
    assert np.array_equal(out[:, :D], v[:, 0, :])
    assert np.allclose(out[:, D:], Z[:, i, j], rtol=1e-6, atol=1e-6)
    want = torch.bmm(torch.from_numpy(v).double(), torch.from_numpy(v).double().transpose(1, 2)).numpy()
    assert np.allclose(out[:, D:], want[:, i, j], rtol=1e-6, atol=1e-6)


def test_interact_orthonormal_and_identical():
    D = 8
    q, _ = np.linalg.qr(rng.normal(size=(D, D)))
    v = q[None, :5, :].astype(np.float32)                   # 5 orthonormal vectors
    out = oracle.interact(v)
    assert np.abs(out[0, D:]).max() < 1e-6
    u = rng.integers(-3, 4, size=D).astype(np.float32)
    out = oracle.interact(np.tile(u, (1, 4, 1)))
    assert np.array_equal(out[0, D:], np.full(6, float(u @ u), np.float32))


# ---------------------------------------------------------------- whole model

def _tiny_model(T=3, R=50, D=8, F=5, integer=False):
    tables = _tables(T, R, D, integer)
    V = T + 1
    pb = synth.mlp_params((F, 12, D), stack=0)
    pt = synth.mlp_params((D + V * (V - 1) // 2, 10, 1), stack=1)
    return tables, pb, pt


def test_model_hand_example(golden):
    g = golden("model_hand_example.txt")
    D, B = int(g["D"][0]), int(g["B"][0])
    tables = [np.array(g["table0"], np.float32).reshape(-1, D)]
    dense = np.array(g["dense"], np.float32).reshape(B, 2)
    Wb, bb = [np.array(g["Wb0"], np.float32).reshape(2, 2)], [np.array(g["bb0"], np.float32)]
    Wt, bt = [np.array(g["Wt0"], np.float32).reshape(1, 3)], [np.array(g["bt0"], np.float32)]
    lengths, idx = np.array(g["lengths"], np.int32), np.array(g["indices"], np.int32)
    x = oracle.fc(dense, Wb[0], bb[0], oracle.ACT_RELU)
    assert x.reshape(-1).tolist() == g["bottom_out"]
    E = oracle.sls(tables, idx, lengths, B)
    assert E.reshape(-1).tolist() == g["E"]
    inter = oracle.interact(np.concatenate([x[:, None, :], E], axis=1))
    assert inter.reshape(-1).tolist() == g["interact"]
    logit = oracle.fc(inter, Wt[0], bt[0], oracle.ACT_NONE)
    assert np.allclose(logit.reshape(-1), g["logit"], rtol=1e-7)
    st, p = oracle.model_forward(tables, Wb, bb, Wt, bt, dense, idx, lengths)
    assert st == oracle.OK
    assert np.allclose(p, g["prob"], rtol=1e-7, atol=0)


def test_model_vs_torch_cpu_float64():
    T, R, D, F, B = 3, 50, 8, 5, 14
    tables, pb, pt = _tiny_model(T, R, D, F)
    dense = rng.uniform(size=(B, F)).astype(np.float32)
    idx, lengths = _bags(T, B, R, 0, 12)
    st, p = oracle.model_forward(tables, pb.W, pb.b, pt.W, pt.b, dense, idx, lengths)
    assert st == oracle.OK and np.all(p > 0) and np.all(p < 1)
    tt = torch.from_numpy
    x = tt(dense).double()
    for W, b in zip(pb.W, pb.b):
        x = torch.relu(torch.nn.functional.linear(x, tt(W).double(), tt(b).double()))
    off = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    vecs = [x]
    for t in range(T):
        lo, hi = off[t * B], off[(t + 1) * B]
        vecs.append(torch.nn.functional.embedding_bag(
            tt(idx[lo:hi].astype(np.int64)), tt(tables[t]).double(), tt(off[t * B:(t + 1) * B] - lo), mode="sum"))
    Vm = torch.stack(vecs, dim=1)
    Z = torch.bmm(Vm, Vm.transpose(1, 2))
    i, j = np.tril_indices(T + 1, -1)
    h = torch.cat([x, Z[:, i, j]], dim=1)
    for l, (W, b) in enumerate(zip(pt.W, pt.b)):
        h = torch.nn.functional.linear(h, tt(W).double(), tt(b).double())
        h = torch.relu(h) if l < len(pt.W) - 1 else torch.sigmoid(h)
    assert np.allclose(p, h.numpy()[:, 0], rtol=2e-6, atol=0)


def test_model_batch_split_and_permutation_invariance():
    T, R, D, F, B = 3, 50, 8, 5, 23
    tables, pb, pt = _tiny_model(T, R, D, F)
    dense = rng.uniform(size=(B, F)).astype(np.float32)
    idx, lengths = _bags(T, B, R, 0, 12)
    st, p = oracle.model_forward(tables, pb.W, pb.b, pt.W, pt.b, dense, idx, lengths)
    assert st == oracle.OK
    off = np.concatenate([[0], np.cumsum(lengths)])

    def take(samples):
        samples = np.asarray(samples)
        L = np.concatenate([lengths[t * B + samples] for t in range(T)])
        I = np.concatenate([idx[off[t * B + b]:off[t * B + b + 1]] for t in range(T) for b in samples]
                           + [np.zeros(0, np.int32)])
        return dense[samples], I.astype(np.int32), L.astype(np.int32)

    # any partition into sub-batches gives the same per-sample result, exactly
    parts = [np.arange(0, 7), np.arange(7, 8), np.arange(8, 23)]
    got = np.concatenate([oracle.model_forward(tables, pb.W, pb.b, pt.W, pt.b, *take(s))[1] for s in parts])
    assert np.array_equal(got, p)
    # permuting samples permutes outputs
    perm = rng.permutation(B)
    assert np.array_equal(oracle.model_forward(tables, pb.W, pb.b, pt.W, pt.b, *take(perm))[1], p[perm])


def test_model_rejects_bad_input():
    tables, pb, pt = _tiny_model()
    dense = rng.uniform(size=(2, 5)).astype(np.float32)
    lengths = np.ones(6, np.int32)
    idx = np.zeros(6, np.int32); idx[4] = 50
    assert oracle.model_forward(tables, pb.W, pb.b, pt.W, pt.b, dense, idx, lengths)[0] == oracle.ERR_INDEX_RANGE
    assert oracle.model_forward(tables, pb.W, pb.b, pt.W, pt.b, dense, idx[:5], lengths)[0] == oracle.ERR_LENGTHS_MISMATCH
    assert oracle.model_forward(tables, pb.W, pb.b, pb.W, pb.b, dense, idx, lengths)[0] == oracle.ERR_BAD_SHAPE


def test_oracle_threads_do_not_change_results():
    T, R, D, F, B = 3, 50, 8, 5, 40
    tables, pb, pt = _tiny_model(T, R, D, F)
    dense = rng.uniform(size=(B, F)).astype(np.float32)
    idx, lengths = _bags(T, B, R, 0, 12)
    oracle.set_threads(1)
    p1 = oracle.model_forward(tables, pb.W, pb.b, pt.W, pt.b, dense, idx, lengths)[1]
    oracle.set_threads(4)
    p4 = oracle.model_forward(tables, pb.W, pb.b, pt.W, pt.b, dense, idx, lengths)[1]
    oracle.set_threads(1)
    assert np.array_equal(p1, p4)


# ---- concatenating models (Table I: NCF / Wide&Deep rows) --------------------------------

def test_concat_model_hand_example(golden):
    g = golden("concat_model_hand_example.txt")
    D, B = int(g["D"][0]), int(g["B"][0])
    tables = [np.array(g[f"table{t}"], np.float32).reshape(-1, D) for t in range(2)]
    dense = np.array(g["dense"], np.float32).reshape(B, 2)
    Wt = [np.array(g["Wt0"], np.float32).reshape(2, 6), np.array(g["Wt1"], np.float32).reshape(1, 2)]
    bt = [np.array(g["bt0"], np.float32), np.array(g["bt1"], np.float32)]
    lengths, idx = np.array(g["lengths"], np.int32), np.array(g["indices"], np.int32)
    E = oracle.sls(tables, idx, lengths, B)
    cat = np.concatenate([dense, E.reshape(B, -1)], axis=1)
    assert cat.reshape(-1).tolist() == g["cat"]
    h = oracle.fc(cat, Wt[0], bt[0], oracle.ACT_RELU)
    assert h.reshape(-1).tolist() == g["hidden"]
    st, p = oracle.model_forward(tables, [], [], Wt, bt, dense, idx, lengths, concat=True)
    assert st == oracle.OK
    assert np.allclose(p, g["prob"], rtol=1e-7, atol=0)


@pytest.mark.parametrize("with_dense_stack", [False, True])
def test_concat_model_vs_torch_cpu_float64(with_dense_stack):
    import torch
    T, R, D, F, B = 5, 40, 4, 6, 11
    tables = [rng.normal(size=(R, D)).astype(np.float32) for _ in range(T)]
    X = 8 if with_dense_stack else F
    pb = synth.mlp_params((F, 10, X), 0, 5) if with_dense_stack else synth.mlp_params((F,), 0, 5)
    pt = synth.mlp_params((X + T * D, 16, 8, 1), 1, 5)
    dense = rng.normal(size=(B, F)).astype(np.float32)
    idx, lengths = _bags(T, B, R, 1, 1)                         # one lookup per table, as in Table I
    if with_dense_stack:
        idx, lengths = _bags(T, B, R, 0, 5)                     # pooled sums are concatenated just the same
    st, p = oracle.model_forward(tables, pb.W, pb.b, pt.W, pt.b, dense, idx, lengths, concat=True)
    assert st == oracle.OK
    # independent formulation: float64 torch ops, rounding to fp32 between layers as the oracle does
    x = torch.from_numpy(dense).double()
    for W, b in zip(pb.W, pb.b):
        x = torch.relu(torch.nn.functional.linear(x, torch.from_numpy(W).double(), torch.from_numpy(b).double())).float().double()
    off = np.concatenate([[0], np.cumsum(lengths)])[:-1].reshape(T, B)
    parts = [x]
    for t in range(T):
        lo, hi = off[t, 0], off[t, 0] + lengths.reshape(T, B)[t].sum()
        e = torch.nn.functional.embedding_bag(torch.from_numpy(idx[lo:hi].astype(np.int64)), torch.from_numpy(tables[t]).double(),
                                              torch.from_numpy((off[t] - off[t, 0]).astype(np.int64)), mode="sum")
        parts.append(e.float().double())
    z = torch.cat(parts, dim=1)
    for i, (W, b) in enumerate(zip(pt.W, pt.b)):
        z = torch.nn.functional.linear(z, torch.from_numpy(W).double(), torch.from_numpy(b).double())
        z = (torch.sigmoid(z) if i == len(pt.W) - 1 else torch.relu(z)).float().double()
    assert np.allclose(p, z.reshape(-1).numpy(), rtol=2e-6, atol=1e-7)


def test_concat_model_shape_errors_and_column_blocks():
    T, R, D, F, B = 3, 20, 4, 4, 6
    tables = [rng.normal(size=(R, D)).astype(np.float32) for _ in range(T)]
    pt = synth.mlp_params((F + T * D, 8, 1), 1, 9)
    dense = rng.normal(size=(B, F)).astype(np.float32)
    idx, lengths = _bags(T, B, R, 1, 1)
    st, p = oracle.model_forward(tables, [], [], pt.W, pt.b, dense, idx, lengths, concat=True)
    assert st == oracle.OK
    # a predictor that ignores the columns of table 1 does not see table 1's indices ...
    W0 = pt.W[0].copy()
    W0[:, F + D:F + 2 * D] = 0
    idx2 = idx.copy()
    idx2[B:2 * B] = (idx2[B:2 * B] + 7) % R
    pa = oracle.model_forward(tables, [], [], [W0] + pt.W[1:], pt.b, dense, idx, lengths, concat=True)[1]
    pb_ = oracle.model_forward(tables, [], [], [W0] + pt.W[1:], pt.b, dense, idx2, lengths, concat=True)[1]
    assert np.array_equal(pa, pb_)
    # ... and the full predictor does
    assert not np.array_equal(p, oracle.model_forward(tables, [], [], pt.W, pt.b, dense, idx2, lengths, concat=True)[1])
    # predictor input width must be dense width + T*D
    bad = synth.mlp_params((F + T * D + 1, 8, 1), 1, 9)
    assert oracle.model_forward(tables, [], [], bad.W, bad.b, dense, idx, lengths, concat=True)[0] == oracle.ERR_BAD_SHAPE
