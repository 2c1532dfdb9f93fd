"""Pins for the oracle's LINE edge sampler.

What the mathematics fixes: every sample is an entry of the graph, the source is
the row that holds the drawn entry (rows without entries are never a source),
the entry index is floor(r * E / 2^64) recomputed with Python integers from the
raw Philox block, uniform and weight-proportional laws (chi-square), the same
stream whether drawn in one call or several, and a stream distinct from the
walker's and the negative sampler's.
"""
import numpy as np
import pytest
import scipy.stats as st


def _csr_with_empty_rows(oracle, seed=0):
    rng = np.random.default_rng(seed)
    n, m = 40, 90
    src = rng.integers(0, n // 2, m).astype(np.int32) * 2      # odd rows stay empty
    dst = rng.integers(0, n, m).astype(np.int32)
    off, nb, _ = oracle.csr_build(src, dst, None, n, oracle.DROP_SELF_LOOPS | oracle.DEDUPE)
    return off, nb


def _entry_index(oracle, seed, i, num_entries):
    key = np.array([seed & 0xFFFFFFFF, seed >> 32], dtype=np.uint32)
    ctr = np.array([i & 0xFFFFFFFF, i >> 32, 0, 0x40000000], dtype=np.uint32)
    x = oracle.philox4x32_10(ctr, key)
    r = (int(x[0]) << 32) | int(x[1])
    return (r * num_entries) >> 64, x


def test_samples_are_entries_with_their_own_row(oracle):
    off, nb = _csr_with_empty_rows(oracle)
    E = len(nb)
    c, o = oracle.sample_edges(off, nb, 500, seed=11)
    for i in range(500):
        e, _ = _entry_index(oracle, 11, i, E)
        row = int(np.searchsorted(off, e, side="right")) - 1
        assert off[row] <= e < off[row + 1]
        assert (int(c[i]), int(o[i])) == (row, int(nb[e]))
    assert (np.diff(off)[c] > 0).all() and (c % 2 == 0).all()


def test_uniform_over_entries(oracle):
    off, nb, _ = oracle.csr_build([0, 0, 1, 2, 3], [1, 2, 2, 3, 0], None, 4, oracle.SYMMETRIZE)
    E = len(nb)
    c, o = oracle.sample_edges(off, nb, 40000, seed=5)
    src = np.repeat(np.arange(4), np.diff(off))
    index = {(int(a), int(b)): e for e, (a, b) in enumerate(zip(src, nb))}
    counts = np.bincount([index[(int(a), int(b))] for a, b in zip(c, o)], minlength=E)
    assert st.chisquare(counts).pvalue > 1e-3
    # every undirected edge appears in both directions
    assert all((b, a) in index for (a, b) in index)


def test_weight_proportional_with_alias_table(oracle):
    src = np.array([0, 0, 1, 2, 2], dtype=np.int32)
    dst = np.array([1, 2, 2, 0, 3], dtype=np.int32)
    w = np.array([1.0, 4.0, 0.5, 2.5, 2.0], dtype=np.float32)
    off, nb, ww = oracle.csr_build(src, dst, w, 4, 0)
    E = len(nb)
    table = oracle.alias_build(np.array([0, E], dtype=np.int64), ww)
    c, o = oracle.sample_edges(off, nb, 60000, seed=9, edge_alias=table)
    srcs = np.repeat(np.arange(4), np.diff(off))
    index = {(int(a), int(b)): e for e, (a, b) in enumerate(zip(srcs, nb))}
    counts = np.bincount([index[(int(a), int(b))] for a, b in zip(c, o)], minlength=E)
    expected = ww.astype(np.float64) / ww.sum() * counts.sum()
    assert st.chisquare(counts, expected).pvalue > 1e-3
    # acceptance uses word 2 of the block: prob[e] against (x2 >> 8) * 2^-24
    prob, alias = table
    for i in range(200):
        e, x = _entry_index(oracle, 9, i, E)
        accept = np.float32(int(x[2]) >> 8) * np.float32(2.0 ** -24)
        e = e if accept < prob[e] else int(alias[e])
        assert (int(c[i]), int(o[i])) == (int(srcs[e]), int(nb[e]))


def test_zero_weight_entries_are_never_drawn(oracle):
    off, nb, ww = oracle.csr_build([0, 0, 1], [1, 2, 2], np.array([0.0, 1.0, 3.0], dtype=np.float32), 3, 0)
    table = oracle.alias_build(np.array([0, len(nb)], dtype=np.int32), ww)
    c, o = oracle.sample_edges(off, nb, 5000, seed=2, edge_alias=table)
    assert not ((c == 0) & (o == 1)).any()
    assert ((c == 0) & (o == 2)).any() and ((c == 1) & (o == 2)).any()


def test_split_calls_and_separate_stream(oracle):
    off, nb = _csr_with_empty_rows(oracle, 3)
    c, o = oracle.sample_edges(off, nb, 300, seed=21)
    c1, o1 = oracle.sample_edges(off, nb, 120, seed=21)
    c2, o2 = oracle.sample_edges(off, nb, 180, seed=21, sample_index_base=120)
    np.testing.assert_array_equal(c, np.concatenate([c1, c2]))
    np.testing.assert_array_equal(o, np.concatenate([o1, o2]))
    # same seed and index, other counter domain: the negative sampler over the same count
    negs = oracle.sample_negatives(None, len(nb), 300, 1, seed=21)[:, 0]
    entry = np.array([_entry_index(oracle, 21, i, len(nb))[0] for i in range(300)])
    assert (negs != entry).mean() > 0.9


def test_line_batch_is_an_sgns_batch_over_edges(oracle):
    """A LINE step (second order) is the SGNS step with the sampled edges as pairs:
    with K negatives a batch of B edges touches at most B * (2 + K) rows."""
    off, nb = _csr_with_empty_rows(oracle, 5)
    n, d, B, K = len(off) - 1, 8, 64, 5
    rng = np.random.default_rng(0)
    w_in = rng.uniform(-0.5, 0.5, (n, d)).astype(np.float32)
    w_out = rng.uniform(-0.5, 0.5, (n, d)).astype(np.float32)
    c, o = oracle.sample_edges(off, nb, B, seed=4)
    negs = oracle.sample_negatives(None, n, B, K, seed=6)
    a, b = w_in.copy(), w_out.copy()
    oracle.sgns_step(a, b, c, o, negs, 0.05)
    touched = set(c.tolist()) | set(o.tolist()) | set(negs.ravel().tolist())
    assert len(touched) <= B * (2 + K)
    same = [r for r in range(n) if r not in touched]
    np.testing.assert_array_equal(a[same], w_in[same])
    np.testing.assert_array_equal(b[same], w_out[same])
    assert not np.array_equal(a[c[0]], w_in[c[0]])


# ----------------------------------------------------------------------------- first order
def _line1_dense(w, s, t, neg):
    import torch
    import torch.nn.functional as F
    ws = w[torch.as_tensor(s, dtype=torch.long)]
    pos = (ws * w[torch.as_tensor(t, dtype=torch.long)]).sum(1)
    ng = (ws[:, None, :] * w[torch.as_tensor(neg, dtype=torch.long)]).sum(2)
    return F.softplus(-pos).sum() + F.softplus(ng).sum()


def test_line1_step_is_sgd_on_one_table(oracle):
    """First-order LINE: both endpoints from the same table.  The step equals dense SGD on
    that table with torch autograd (rows on both sides get both gradient parts; a pair with
    s == t or a negative equal to the source is differentiated through both factors)."""
    import torch
    rng = np.random.default_rng(3)
    n, d, b, k, lr = 25, 6, 80, 3, 0.05
    w = rng.normal(0, 0.5, (n, d)).astype(np.float32)
    s = rng.integers(0, 15, b).astype(np.int32)           # rows 15.. are never a source
    t = rng.integers(0, 20, b).astype(np.int32)           # rows 20.. are never named
    neg = rng.integers(0, 20, (b, k)).astype(np.int32)
    t[:5] = s[:5]                                         # self pairs
    neg[5:10, 0] = s[5:10]                                # the source among its negatives
    tw = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    dense = _line1_dense(tw, s, t, neg)
    dense.backward()
    want = w.astype(np.float64) - np.float64(np.float32(lr)) * tw.grad.numpy()
    got = w.copy()
    loss = oracle.line1_step(got, s, t, neg, lr)
    assert loss == pytest.approx(dense.item(), rel=1e-12)
    np.testing.assert_allclose(got, want, atol=2e-7)      # two fp32 roundings per element at most
    np.testing.assert_array_equal(got[20:], w[20:])


def test_line1_step_writes_in_two_rounds(oracle):
    """bf16 table: a row that is both a source and a target is rounded after the
    contributions it gets as target/negative and again after those it gets as source."""
    import torch
    w = np.array([[1.0, 0.5], [0.25, -1.0], [2.0, 1.0]], dtype=np.float32)
    bits = torch.from_numpy(w).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy()
    s = np.array([0, 1], dtype=np.int32)
    t = np.array([1, 0], dtype=np.int32)
    neg = np.zeros((2, 0), dtype=np.int32)
    lr = 0.3
    sig = lambda x: 1.0 / (1.0 + np.exp(-x))
    x = float(w[0] @ w[1])
    g = sig(x) - 1.0
    to_bf16 = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float32)).to(torch.bfloat16).to(torch.float32).numpy()
    lr32 = np.float64(np.float32(lr))
    # row 0: as target of pair (1, 0): g * w[1]; as source of pair (0, 1): g * w[1]
    r0 = to_bf16(to_bf16(w[0] - lr32 * g * w[1]) - lr32 * g * w[1])
    r1 = to_bf16(to_bf16(w[1] - lr32 * g * w[0]) - lr32 * g * w[0])
    oracle.line1_step(bits, s, t, neg, lr, dtype=oracle.BF16)
    got = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(got[0], r0)
    np.testing.assert_array_equal(got[1], r1)
    np.testing.assert_array_equal(got[2], w[2])


def test_line1_round_order_target_part_first(oracle):
    """Row 0 is the source of pair (0, 1) and the target of pair (2, 0): it is rounded after
    its target part and again after its source part.  Recomputed by hand with torch's bf16
    rounding; the values are chosen so that the opposite order gives another result."""
    import torch
    rng = np.random.default_rng(12)
    to_bf16 = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float32)).to(torch.bfloat16).to(torch.float32).numpy()
    sig = lambda x: 1.0 / (1.0 + np.exp(-x))
    for trial in range(50):
        w = to_bf16(rng.normal(0, 1.0, (3, 4))).astype(np.float64)
        lr = np.float64(np.float32(0.37))
        g1 = sig(w[0] @ w[1]) - 1.0          # pair (0, 1)
        g2 = sig(w[2] @ w[0]) - 1.0          # pair (2, 0)
        as_target = g2 * w[2]
        as_source = g1 * w[1]
        right = to_bf16(to_bf16(w[0] - lr * as_target).astype(np.float64) - lr * as_source)
        wrong = to_bf16(to_bf16(w[0] - lr * as_source).astype(np.float64) - lr * as_target)
        if not np.array_equal(right, wrong):
            break
    else:
        raise AssertionError("no discriminating case found")
    bits = torch.from_numpy(w.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy()
    oracle.line1_step(bits, np.array([0, 2], dtype=np.int32), np.array([1, 0], dtype=np.int32),
                      np.zeros((2, 0), dtype=np.int32), 0.37, dtype=oracle.BF16)
    got = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(got[0], right)
