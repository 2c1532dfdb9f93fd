"""Pins for the oracle's walkers, pair emission and negative sampler.

Checks against things the mathematics fixes: every step is an edge, forced
walks, uniformity on a complete graph, the degree-proportional stationary
distribution, the node2vec transition law by brute-force enumeration, closed
form pair counts, brute-force pair lists, and chi-square tests of the noise
distribution.
"""
import itertools

import numpy as np
import pytest
import scipy.stats as st


def _graph(oracle, n, m, seed, directed=False):
    rng = np.random.default_rng(seed)
    src = rng.integers(0, n, m).astype(np.int32)
    dst = rng.integers(0, n, m).astype(np.int32)
    flags = oracle.DROP_SELF_LOOPS | oracle.DEDUPE | (0 if directed else oracle.SYMMETRIZE)
    off, nb, _ = oracle.csr_build(src, dst, None, n, flags)
    return off, nb


def _edge_set(off, nb):
    return {(v, int(x)) for v in range(len(off) - 1) for x in nb[off[v]:off[v + 1]]}


def _assert_walks_valid(walks, off, nb, starts):
    edges = _edge_set(off, nb)
    deg = np.diff(off)
    for row, s in zip(walks, starts):
        assert row[0] == s
        for t in range(len(row) - 1):
            a, b = int(row[t]), int(row[t + 1])
            if a < 0 or deg[a] == 0:
                assert b == -1
            else:
                assert (a, b) in edges


# ----------------------------------------------------------------------------- first order
def test_walk_steps_are_edges_and_dead_ends_pad(oracle):
    off, nb = _graph(oracle, 60, 150, 1, directed=True)
    assert (np.diff(off) == 0).any()          # the directed graph has sinks
    starts = np.arange(60, dtype=np.int32).repeat(5)
    walks = oracle.random_walk(off, nb, starts, 12, seed=3)
    _assert_walks_valid(walks, off, nb, starts)
    assert (walks == -1).any()


def test_walk_two_node_graph_is_forced(oracle):
    off, nb, _ = oracle.csr_build([0], [1], None, 2, oracle.SYMMETRIZE)
    walks = oracle.random_walk(off, nb, [0, 1], 7, seed=5)
    np.testing.assert_array_equal(walks, [[0, 1, 0, 1, 0, 1, 0], [1, 0, 1, 0, 1, 0, 1]])


def test_walk_len_one_and_bad_start(oracle):
    off, nb = _graph(oracle, 10, 30, 2)
    walks = oracle.random_walk(off, nb, [3, 4], 1, seed=1)
    np.testing.assert_array_equal(walks, [[3], [4]])
    walks = oracle.random_walk(off, nb, [-5, 10], 3, seed=1)
    assert (walks == -1).all()


def test_walk_is_uniform_on_complete_graph(oracle):
    n = 9
    src, dst = zip(*[(a, b) for a in range(n) for b in range(n) if a != b])
    off, nb, _ = oracle.csr_build(src, dst, None, n, oracle.DEDUPE)
    walks = oracle.random_walk(off, nb, np.zeros(60_000, dtype=np.int32), 3, seed=17)
    first = np.bincount(walks[:, 1], minlength=n)
    assert first[0] == 0
    assert st.chisquare(first[1:]).pvalue > 0.01
    # second step, conditioned on the first being node 4
    second = np.bincount(walks[walks[:, 1] == 4][:, 2], minlength=n)
    assert second[4] == 0
    assert st.chisquare(np.delete(second, 4)).pvalue > 0.01


def test_walk_stationary_distribution_is_degree_proportional(oracle):
    off, nb = _graph(oracle, 40, 160, 4)
    deg = np.diff(off).astype(np.float64)
    assert deg.min() > 0
    rng = np.random.default_rng(8)
    starts = rng.choice(40, size=120_000, p=deg / deg.sum()).astype(np.int32)
    walks = oracle.random_walk(off, nb, starts, 6, seed=23)
    # only the last node of each walk: independent samples of the stationary law
    counts = np.bincount(walks[:, -1], minlength=40)
    assert st.chisquare(counts, counts.sum() * deg / deg.sum()).pvalue > 0.01


def test_walk_split_calls_match_one_call(oracle):
    off, nb = _graph(oracle, 50, 200, 6)
    starts = (np.arange(300) % 50).astype(np.int32)
    whole = oracle.random_walk(off, nb, starts, 9, seed=77)
    a = oracle.random_walk(off, nb, starts[:101], 9, seed=77, walk_id_base=0)
    b = oracle.random_walk(off, nb, starts[101:], 9, seed=77, walk_id_base=101)
    np.testing.assert_array_equal(whole, np.vstack([a, b]))
    other = oracle.random_walk(off, nb, starts, 9, seed=78)
    assert (other != whole).any()


def test_weighted_walk_follows_edge_weights(oracle):
    # star: node 0 -> leaves 1..5 with weights 1..5 (directed, leaves are sinks)
    src = np.zeros(5, dtype=np.int32)
    dst = np.arange(1, 6, dtype=np.int32)
    w = np.arange(1, 6, dtype=np.float32)
    off, nb, wo = oracle.csr_build(src, dst, w, 6, 0)
    table = oracle.alias_build(off, wo)
    walks = oracle.random_walk(off, nb, np.zeros(100_000, dtype=np.int32), 2, seed=9, alias=table)
    counts = np.bincount(walks[:, 1], minlength=6)[1:]
    assert st.chisquare(counts, counts.sum() * w / w.sum()).pvalue > 0.01


# ----------------------------------------------------------------------------- node2vec
def test_node2vec_with_unit_bias_equals_first_order_walk(oracle):
    off, nb = _graph(oracle, 80, 400, 11)
    starts = (np.arange(500) % 80).astype(np.int32)
    a = oracle.random_walk(off, nb, starts, 15, seed=5)
    b = oracle.node2vec_walk(off, nb, starts, 15, 1.0, 1.0, seed=5)
    np.testing.assert_array_equal(a, b)
    # same with per-row alias tables
    rng = np.random.default_rng(0)
    table = oracle.alias_build(off, rng.random(nb.size).astype(np.float32) + 0.1)
    a = oracle.random_walk(off, nb, starts, 15, seed=5, alias=table)
    b = oracle.node2vec_walk(off, nb, starts, 15, 1.0, 1.0, seed=5, alias=table)
    np.testing.assert_array_equal(a, b)


@pytest.mark.parametrize("p,q", [(0.5, 2.0), (4.0, 0.25)])
def test_node2vec_transition_law_by_enumeration(oracle, p, q):
    off, nb = _graph(oracle, 12, 30, 13)
    edges = _edge_set(off, nb)
    n = 12
    nw = 400_000
    starts = (np.arange(nw) % n).astype(np.int32)
    walks = oracle.node2vec_walk(off, nb, starts, 3, p, q, seed=31)
    _assert_walks_valid(walks, off, nb, starts)
    tested = 0
    for prev in range(n):
        for cur in nb[off[prev]:off[prev + 1]]:
            cur = int(cur)
            sel = walks[(walks[:, 0] == prev) & (walks[:, 1] == cur)][:, 2]
            cand = [int(x) for x in nb[off[cur]:off[cur + 1]]]
            if len(cand) < 2 or len(sel) < 200:
                continue
            bias = np.array([1 / p if x == prev else (1.0 if (prev, x) in edges else 1 / q)
                             for x in cand])
            counts = np.array([(sel == x).sum() for x in cand])
            assert counts.sum() == len(sel)
            pv = st.chisquare(counts, len(sel) * bias / bias.sum()).pvalue
            assert pv > 1e-4, (prev, cur, counts, bias)   # ~60 tests: Bonferroni-style floor
            tested += 1
    assert tested >= 20


def test_node2vec_weighted_transition_law(oracle):
    rng = np.random.default_rng(3)
    n = 8
    src, dst = zip(*[(a, b) for a in range(n) for b in range(a + 1, n) if rng.random() < 0.6])
    w = (rng.random(len(src)) * 3 + 0.2).astype(np.float32)
    off, nb, wo = oracle.csr_build(src, dst, w, n, oracle.SYMMETRIZE)
    edges = _edge_set(off, nb)
    table = oracle.alias_build(off, wo)
    p, q = 0.5, 2.0
    nw = 300_000
    walks = oracle.node2vec_walk(off, nb, (np.arange(nw) % n).astype(np.int32), 3, p, q,
                                 seed=41, alias=table)
    tested = 0
    for prev in range(n):
        for cur in nb[off[prev]:off[prev + 1]]:
            cur = int(cur)
            sel = walks[(walks[:, 0] == prev) & (walks[:, 1] == cur)][:, 2]
            cand = [int(x) for x in nb[off[cur]:off[cur + 1]]]
            if len(cand) < 2 or len(sel) < 500:
                continue
            ew = wo[off[cur]:off[cur + 1]].astype(np.float64)
            bias = np.array([1 / p if x == prev else (1.0 if (prev, x) in edges else 1 / q)
                             for x in cand]) * ew
            counts = np.array([(sel == x).sum() for x in cand])
            assert st.chisquare(counts, len(sel) * bias / bias.sum()).pvalue > 1e-4
            tested += 1
    assert tested >= 10


def test_node2vec_directed_membership_uses_prev_row(oracle):
    # 0->1, 1->2, 1->3, 0->2 (directed).  From prev=0, cur=1: x=2 is a neighbour
    # of prev (bias 1), x=3 is not (bias 1/q).
    off, nb, _ = oracle.csr_build([0, 1, 1, 0], [1, 2, 3, 2], None, 4, 0)
    q = 4.0
    walks = oracle.node2vec_walk(off, nb, np.zeros(80_000, dtype=np.int32), 3, 1.0, q, seed=2)
    sel = walks[walks[:, 1] == 1][:, 2]
    c2, c3 = (sel == 2).sum(), (sel == 3).sum()
    assert c2 + c3 == len(sel)
    assert st.chisquare([c2, c3], [len(sel) * 0.8, len(sel) * 0.2]).pvalue > 0.01


def test_node2vec_rejects_bad_parameters(oracle):
    off, nb = _graph(oracle, 10, 30, 2)
    with pytest.raises(ValueError):
        oracle.node2vec_walk(off, nb, [0], 3, 0.0, 1.0, seed=1)
    with pytest.raises(ValueError):
        oracle.node2vec_walk(off, nb, [0], 3, 1.0, -1.0, seed=1)


# ----------------------------------------------------------------------------- pairs
def _brute_pairs(walks, window):
    out = []
    for row in walks:
        row = list(row)
        length = row.index(-1) if -1 in row else len(row)
        for a in range(length):
            for b in range(max(0, a - window), min(length, a + window + 1)):
                if b != a:
                    out.append((row[a], row[b]))
    return out


@pytest.mark.parametrize("walk_len,window", [(20, 5), (5, 3), (4, 7), (1, 2), (40, 5), (80, 10)])
def test_pair_count_closed_form(oracle, walk_len, window):
    walks = np.arange(3 * walk_len, dtype=np.int32).reshape(3, walk_len)
    c, _ = oracle.make_pairs(walks, window)
    if walk_len > window:
        per = 2 * window * walk_len - window * (window + 1)
    else:
        per = walk_len * (walk_len - 1)
    assert len(c) == 3 * per


def test_pair_counts_at_the_five_workloads(oracle):
    for (walk_len, window), want in {(20, 5): 170, (40, 5): 370, (80, 10): 1490}.items():
        c, _ = oracle.make_pairs(np.zeros((1, walk_len), dtype=np.int32), window)
        assert len(c) == want


def test_pairs_match_brute_force_with_dead_ends(oracle):
    rng = np.random.default_rng(12)
    walks = rng.integers(0, 50, (40, 11)).astype(np.int32)
    for i in range(40):
        cut = rng.integers(1, 14)
        if cut < 11:
            walks[i, cut:] = -1
    walks[7, :] = -1
    for window in (1, 3, 12):
        c, o = oracle.make_pairs(walks, window)
        assert list(zip(c.tolist(), o.tolist())) == _brute_pairs(walks, window)


def test_pair_multiset_is_symmetric(oracle):
    rng = np.random.default_rng(14)
    walks = rng.integers(0, 6, (1, 30)).astype(np.int32)
    c, o = oracle.make_pairs(walks, 4)
    fwd = sorted(zip(c.tolist(), o.tolist()))
    rev = sorted(zip(o.tolist(), c.tolist()))
    assert fwd == rev


# ----------------------------------------------------------------------------- negatives
def test_negatives_follow_noise_distribution(oracle):
    off, nb = _graph(oracle, 30, 60, 21)
    deg = np.diff(off).astype(np.float64)
    w = np.where(deg > 0, deg ** 0.75, 0).astype(np.float32)
    assert (w == 0).any()
    table = oracle.alias_build(np.array([0, 30], dtype=np.int32), w)
    negs = oracle.sample_negatives(table, 30, 60_000, 5, seed=4)
    counts = np.bincount(negs.ravel(), minlength=30)
    assert counts[w == 0].sum() == 0
    keep = w > 0
    wd = w.astype(np.float64)
    assert st.chisquare(counts[keep], counts.sum() * wd[keep] / wd.sum()).pvalue > 0.01
    # the k draws of one pair are not copies of each other
    assert (negs[:, 0] != negs[:, 1]).mean() > 0.5


def test_negatives_uniform_when_no_table(oracle):
    negs = oracle.sample_negatives(None, 10, 50_000, 2, seed=6)
    assert st.chisquare(np.bincount(negs.ravel(), minlength=10)).pvalue > 0.01


def test_negatives_are_independent_of_batching(oracle):
    w = np.arange(1, 41, dtype=np.float32)
    table = oracle.alias_build(np.array([0, 40], dtype=np.int32), w)
    whole = oracle.sample_negatives(table, 40, 1000, 5, seed=8)
    a = oracle.sample_negatives(table, 40, 333, 5, seed=8, pair_index_base=0)
    b = oracle.sample_negatives(table, 40, 667, 5, seed=8, pair_index_base=333)
    np.testing.assert_array_equal(whole, np.vstack([a, b]))


def test_walk_and_negative_streams_differ(oracle):
    # same seed, same indices: the tag in the counter keeps the two streams apart
    off, nb, _ = oracle.csr_build(np.zeros(16, dtype=np.int32), np.arange(1, 17, dtype=np.int32),
                                  None, 17, 0)
    walks = oracle.random_walk(off, nb, np.zeros(200, dtype=np.int32), 2, seed=1)
    negs = oracle.sample_negatives(None, 16, 200, 1, seed=1)
    assert (walks[:, 1] - 1 != negs[:, 0]).any()


def test_slot_matches_integer_arithmetic(oracle):
    # uniform neighbour = floor(r * deg / 2**64) for the 64-bit r of words 0,1:
    # recompute with Python integers from the raw block
    off, nb, _ = oracle.csr_build(np.zeros(1000, dtype=np.int32),
                                  np.arange(1, 1001, dtype=np.int32), None, 1001, 0)
    walks = oracle.random_walk(off, nb, np.zeros(50, dtype=np.int32), 2, seed=0xABCDEF0123456789,
                               walk_id_base=(1 << 33) + 5)
    for i in range(50):
        wid = (1 << 33) + 5 + i
        blk = oracle.philox4x32_10([wid & 0xFFFFFFFF, wid >> 32, 0, 0],
                                   [0x23456789, 0xABCDEF01])
        r = (int(blk[0]) << 32) | int(blk[1])
        assert walks[i, 1] == 1 + ((r * 1000) >> 64)
