"""Property tests of the oracle against brute force / numpy on random small inputs
(hypothesis): pair emission, merged ids, pair sorting, alias tables."""
from fractions import Fraction

import numpy as np
from hypothesis import given, settings, strategies as st


@settings(max_examples=60, deadline=None, derandomize=True)
@given(st.integers(1, 12), st.integers(1, 6), st.integers(0, 6), st.integers(0, 2 ** 31 - 1))
def test_make_pairs_matches_brute_force(oracle, walk_len, window, num_walks, seed):
    rng = np.random.default_rng(seed)
    walks = rng.integers(0, 50, (num_walks, walk_len)).astype(np.int32)
    for i in range(num_walks):                              # dead ends: -1 as a suffix
        cut = rng.integers(0, walk_len + 1)
        walks[i, cut:] = -1
    want = []
    for row in walks:
        valid = int((row >= 0).sum())
        for a in range(valid):
            for b in range(-window, window + 1):
                if b != 0 and 0 <= a + b < valid:
                    want.append((int(row[a]), int(row[a + b])))
    c, o = oracle.make_pairs(walks, window)
    assert list(zip(c.tolist(), o.tolist())) == want


@settings(max_examples=60, deadline=None, derandomize=True)
@given(st.lists(st.integers(-3, 40), max_size=80), st.integers(1, 38))
def test_unique_ids_matches_numpy(oracle, ids, num_nodes):
    ids = np.array(ids, dtype=np.int32)
    u, inv = oracle.unique_ids(ids, num_nodes)
    ok = (ids >= 0) & (ids < num_nodes)
    wu = np.unique(ids[ok])
    np.testing.assert_array_equal(u, wu)
    assert (inv[~ok] == -1).all()
    np.testing.assert_array_equal(u[inv[ok]], ids[ok])


@settings(max_examples=60, deadline=None, derandomize=True)
@given(st.lists(st.tuples(st.integers(-2, 20), st.integers(0, 1000)), max_size=60), st.integers(1, 19))
def test_sort_pairs_is_stable(oracle, pairs, num_nodes):
    c = np.array([p[0] for p in pairs], dtype=np.int32)
    o = np.array([p[1] for p in pairs], dtype=np.int32)
    sc, so = oracle.sort_pairs(c, o, num_nodes)
    key = np.where((c >= 0) & (c < num_nodes), c, num_nodes)
    order = np.argsort(key, kind="stable")
    np.testing.assert_array_equal(sc, c[order])
    np.testing.assert_array_equal(so, o[order])


@settings(max_examples=40, deadline=None, derandomize=True)
@given(st.lists(st.floats(0, 1e3, width=32), min_size=1, max_size=24))
def test_alias_table_implies_the_weights(oracle, weights):
    w = np.array(weights, dtype=np.float32)
    if float(w.sum()) <= 0:
        w[0] = 1.0
    n = w.size
    prob, alias = oracle.alias_build(np.array([0, n], dtype=np.int32), w)
    mass = [Fraction(0)] * n
    for i in range(n):
        p = Fraction(float(prob[i]))
        mass[i] += p
        mass[int(alias[i])] += 1 - p
    total = sum(Fraction(float(x)) for x in w)
    for i in range(n):
        want = Fraction(float(w[i])) * n / total
        assert abs(mass[i] - want) <= Fraction(n, 2 ** 22)      # n roundings of prob to fp32
    assert all(0 <= int(a) < n for a in alias) and all(0.0 <= float(p) <= 1.0 for p in prob)
