"""Pins for the oracle's storage operations on a batch of ids (unique / get / put).

They reduce to library routines: numpy.unique with its inverse, fancy indexing,
numpy.add.at; bf16 through torch's conversions.  Together they give the sparse
update the paper describes: a put of summed gradient rows onto the distinct ids
of a batch equals the dense update with a gradient that is zero elsewhere.
"""
import numpy as np
import pytest
import torch


def _bf16_bits(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def _bf16_vals(bits):
    return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()


def test_unique_matches_numpy(oracle):
    rng = np.random.default_rng(0)
    ids = rng.integers(0, 50, 400).astype(np.int32)
    u, inv = oracle.unique_ids(ids, 50)
    wu, winv = np.unique(ids, return_inverse=True)
    np.testing.assert_array_equal(u, wu)
    np.testing.assert_array_equal(inv, winv)
    np.testing.assert_array_equal(u[inv], ids)


def test_unique_edge_cases(oracle):
    u, inv = oracle.unique_ids(np.zeros(0, dtype=np.int32), 5)
    assert u.size == 0 and inv.size == 0
    u, inv = oracle.unique_ids([4, 4, 4], 5)
    np.testing.assert_array_equal(u, [4]); np.testing.assert_array_equal(inv, [0, 0, 0])
    u, inv = oracle.unique_ids([7, -3, 2, 5, 2, 9], 6)          # 7, -3, 9 are not rows
    np.testing.assert_array_equal(u, [2, 5]); np.testing.assert_array_equal(inv, [-1, -1, 0, 1, 0, -1])


def test_get_is_fancy_indexing(oracle):
    rng = np.random.default_rng(1)
    t = rng.normal(size=(30, 6)).astype(np.float32)
    ids = np.array([3, 29, 3, 0, 30, -1], dtype=np.int32)
    got = oracle.get_rows(t, ids)
    np.testing.assert_array_equal(got[:4], t[ids[:4]])
    assert (got[4:] == 0).all()
    bits = _bf16_bits(t)
    got = oracle.get_rows(bits, ids, dtype=oracle.BF16)
    np.testing.assert_array_equal(got[:4], _bf16_vals(bits)[ids[:4]])


def test_put_is_add_at(oracle):
    rng = np.random.default_rng(2)
    t = rng.normal(size=(40, 5)).astype(np.float32)
    ids = rng.permutation(40)[:17].astype(np.int32)
    rows = rng.normal(size=(17, 5)).astype(np.float32)
    want = t.astype(np.float64)
    np.add.at(want, ids, -0.25 * rows.astype(np.float64))
    got = t.copy()
    oracle.put_rows(got, ids, rows, -0.25)
    np.testing.assert_array_equal(got, want.astype(np.float32))
    untouched = np.setdiff1d(np.arange(40), ids)
    np.testing.assert_array_equal(got[untouched], t[untouched])
    # ids that are not rows are skipped, duplicates are refused
    got2 = t.copy()
    oracle.put_rows(got2, np.array([1, 40, -2], dtype=np.int32), rows[:3], 1.0)
    np.testing.assert_array_equal(got2[1], (t[1].astype(np.float64) + rows[0]).astype(np.float32))
    np.testing.assert_array_equal(np.delete(got2, 1, 0), np.delete(t, 1, 0))
    with pytest.raises(ValueError):
        oracle.put_rows(t.copy(), np.array([1, 1], dtype=np.int32), rows[:2], 1.0)


def test_put_bf16_rounds_once(oracle):
    rng = np.random.default_rng(3)
    t = rng.normal(size=(20, 8)).astype(np.float32)
    bits = _bf16_bits(t)
    ids = np.array([0, 19, 7], dtype=np.int32)
    rows = rng.normal(size=(3, 8)).astype(np.float32)
    want = _bf16_vals(bits).astype(np.float64)
    want[ids] += 0.5 * rows.astype(np.float64)
    got = bits.copy()
    oracle.put_rows(got, ids, rows, 0.5, dtype=oracle.BF16)
    np.testing.assert_array_equal(got, _bf16_bits(want.astype(np.float32)))


def test_unique_get_put_give_the_sparse_sgd_step(oracle):
    """get the distinct rows, compute on the n x d block, put the summed deltas:
    the result equals the SGNS step on the full tables (the paper's sparse update)."""
    rng = np.random.default_rng(4)
    n, d, B, K = 60, 4, 32, 3
    w_in = rng.uniform(-0.5, 0.5, (n, d)).astype(np.float32)
    w_out = rng.uniform(-0.5, 0.5, (n, d)).astype(np.float32)
    c = rng.integers(0, n, B).astype(np.int32)
    o = rng.integers(0, n, B).astype(np.int32)
    neg = rng.integers(0, n, (B, K)).astype(np.int32)
    full_in, full_out = w_in.copy(), w_out.copy()
    oracle.sgns_step(full_in, full_out, c, o, neg, 0.1)
    # the same through the block: ids of the batch, compacted tables, local step, put of the deltas
    ids = np.concatenate([c, o, neg.ravel()])
    u, inv = oracle.unique_ids(ids, n)
    blk_in, blk_out = oracle.get_rows(w_in, u), oracle.get_rows(w_out, u)
    new_in, new_out = blk_in.copy(), blk_out.copy()
    oracle.sgns_step(new_in, new_out, inv[:B], inv[B:2 * B], inv[2 * B:].reshape(B, K), 0.1)
    got_in, got_out = w_in.copy(), w_out.copy()
    oracle.put_rows(got_in, u, new_in.astype(np.float64) - blk_in, 1.0)
    oracle.put_rows(got_out, u, new_out.astype(np.float64) - blk_out, 1.0)
    np.testing.assert_allclose(got_in, full_in, atol=1e-6)
    np.testing.assert_allclose(got_out, full_out, atol=1e-6)


def test_dense_mult_and_mult_add(oracle):
    rng = np.random.default_rng(5)
    a = rng.normal(size=(7, 5)).astype(np.float32)
    b = rng.normal(size=(7, 5)).astype(np.float32)
    got = a.copy()
    oracle.table_mult(got, 0.9)
    np.testing.assert_array_equal(got, (a.astype(np.float64) * np.float64(np.float32(0.9))).astype(np.float32))
    got = a.copy()
    oracle.table_mult_add(got, b, -0.05)
    want = a.astype(np.float64) + np.float64(np.float32(-0.05)) * b.astype(np.float64)
    np.testing.assert_array_equal(got, want.astype(np.float32))
    ba, bb = _bf16_bits(a), _bf16_bits(b)
    got = ba.copy()
    oracle.table_mult_add(got, bb, 0.5, dtype=oracle.BF16)
    want = _bf16_vals(ba).astype(np.float64) + 0.5 * _bf16_vals(bb).astype(np.float64)
    np.testing.assert_array_equal(got, _bf16_bits(want.astype(np.float32)))


def test_momentum_step_is_mult_put_mult_add(oracle):
    """The paper's model update composed from the storage operations: mult on the momentum,
    put of the batch's gradient rows, mult_add onto the model, equals the momentum step."""
    rng = np.random.default_rng(6)
    n, d, b, k, lr, mu = 40, 6, 50, 3, 0.05, 0.9
    w_in = rng.normal(0, 0.5, (n, d)).astype(np.float32)
    w_out = rng.normal(0, 0.5, (n, d)).astype(np.float32)
    m_in = rng.normal(0, 0.1, (n, d)).astype(np.float32)
    m_out = rng.normal(0, 0.1, (n, d)).astype(np.float32)
    c = rng.integers(0, n, b).astype(np.int32)
    o = rng.integers(0, n, b).astype(np.int32)
    neg = rng.integers(0, n, (b, k)).astype(np.int32)
    want = [t.copy() for t in (w_in, w_out, m_in, m_out)]
    oracle.sgns_momentum_step(*want, c, o, neg, lr, mu)
    # gradient rows from a plain step with lr = 1: old - new
    s_in, s_out = w_in.copy(), w_out.copy()
    oracle.sgns_step(s_in, s_out, c, o, neg, 1.0)
    got = [t.copy() for t in (w_in, w_out, m_in, m_out)]
    for model, moment, stepped, before in ((got[0], got[2], s_in, w_in), (got[1], got[3], s_out, w_out)):
        oracle.table_mult(moment, mu)
        rows, _ = oracle.unique_ids(np.nonzero((stepped != before).any(1))[0].astype(np.int32), n)
        oracle.put_rows(moment, rows, before[rows].astype(np.float64) - stepped[rows], 1.0)
        oracle.table_mult_add(model, moment, -lr)
    for g, w in zip(got, want):
        np.testing.assert_allclose(g, w, atol=1e-6)


def test_sort_pairs_is_a_stable_argsort(oracle):
    rng = np.random.default_rng(7)
    c = rng.integers(0, 30, 500).astype(np.int32)
    o = rng.integers(0, 1000, 500).astype(np.int32)
    c[[3, 77]] = [-1, 30]                                  # not rows: last, in input order
    sc, so = oracle.sort_pairs(c, o, 30)
    key = np.where((c >= 0) & (c < 30), c, 30)
    order = np.argsort(key, kind="stable")
    np.testing.assert_array_equal(sc, c[order])
    np.testing.assert_array_equal(so, o[order])
    assert list(sc[-2:]) == [-1, 30]


def test_sorting_a_batch_does_not_change_the_step(oracle):
    rng = np.random.default_rng(8)
    n, d, b, k = 30, 4, 200, 3
    w_in = rng.normal(0, 0.5, (n, d)).astype(np.float32)
    w_out = rng.normal(0, 0.5, (n, d)).astype(np.float32)
    c = rng.integers(0, n, b).astype(np.int32)
    o = rng.integers(0, n, b).astype(np.int32)
    neg = rng.integers(0, n, (b, k)).astype(np.int32)
    a_in, a_out = w_in.copy(), w_out.copy()
    la = oracle.sgns_step(a_in, a_out, c, o, neg, 0.05)
    # the same multiset of (centre, context, negatives) triples in sorted order
    order = np.argsort(c, kind="stable")
    sc, so = oracle.sort_pairs(c, o, n)
    np.testing.assert_array_equal(sc, c[order])
    b_in, b_out = w_in.copy(), w_out.copy()
    lb = oracle.sgns_step(b_in, b_out, sc, so, neg[order], 0.05)
    assert la == pytest.approx(lb, rel=1e-12)
    np.testing.assert_allclose(a_in, b_in, atol=1e-7)
    np.testing.assert_allclose(a_out, b_out, atol=1e-7)
