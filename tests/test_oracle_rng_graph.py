"""Pins for the oracle's random numbers, CSR construction and alias tables.

Each check compares the oracle with something that is not the oracle: published
known-answer vectors, a library routine (scipy.sparse), brute force in Python,
hand-computed tables, exact rational arithmetic, or a chi-square test.
"""
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.sparse as sp
import scipy.stats as st

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- Philox
def test_philox_known_answers(oracle):
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        out = oracle.philox4x32_10(v[0:4], v[4:6])
        assert [int(x) for x in out] == v[6:10]


def test_philox_is_a_bijection_of_the_counter(oracle):
    # a block cipher in the counter: distinct counters give distinct blocks
    seen = set()
    for c in range(2000):
        seen.add(tuple(int(x) for x in oracle.philox4x32_10([c, 0, 0, 0], [7, 9])))
    assert len(seen) == 2000


def test_philox_words_are_uniform(oracle):
    words = np.array([oracle.philox4x32_10([c, 1, 2, 3], [11, 13]) for c in range(4000)])
    for col in range(4):
        counts = np.bincount(words[:, col] >> 28, minlength=16)
        assert st.chisquare(counts).pvalue > 1e-3


# ----------------------------------------------------------------------------- CSR
def _brute_csr(src, dst, w, n, sym, noself, dedupe):
    ent = []
    for i, (s, d) in enumerate(zip(src, dst)):
        if not (0 <= s < n and 0 <= d < n):
            continue
        if noself and s == d:
            continue
        ent.append((s, d, i))
        if sym:
            ent.append((d, s, i))
    ent.sort()
    out = []
    for e in ent:
        if dedupe and out and out[-1][0] == e[0] and out[-1][1] == e[1]:
            continue
        out.append(e)
    offsets = np.zeros(n + 1, dtype=np.int64)
    for s, _, _ in out:
        offsets[s + 1] += 1
    return np.cumsum(offsets), np.array([e[1] for e in out], dtype=np.int32), \
        None if w is None else np.array([w[e[2]] for e in out], dtype=np.float32)


@pytest.mark.parametrize("flags", range(8))
@pytest.mark.parametrize("bits", [32, 64])
def test_csr_build_matches_brute_force(oracle, flags, bits):
    rng = np.random.default_rng(100 + flags)
    n, m = 23, 300
    src = rng.integers(-1, n + 1, m).astype(np.int32)   # includes out-of-range ids
    dst = rng.integers(-1, n + 1, m).astype(np.int32)
    w = rng.random(m).astype(np.float32)
    off, nb, wo = oracle.csr_build(src, dst, w, n, flags, bits)
    eo, en, ew = _brute_csr(src, dst, w, n, flags & 1, flags & 2, flags & 4)
    assert off.dtype == (np.int64 if bits == 64 else np.int32)
    np.testing.assert_array_equal(off, eo)
    np.testing.assert_array_equal(nb, en)
    np.testing.assert_array_equal(wo, ew)


def test_csr_build_matches_scipy(oracle):
    rng = np.random.default_rng(5)
    n, m = 200, 5000
    src = rng.integers(0, n, m).astype(np.int32)
    dst = rng.integers(0, n, m).astype(np.int32)
    off, nb, _ = oracle.csr_build(src, dst, None, n, oracle.SYMMETRIZE | oracle.DEDUPE
                                  | oracle.DROP_SELF_LOOPS)
    a = sp.coo_matrix((np.ones(m), (src, dst)), shape=(n, n)).tocsr()
    a = a + a.T
    a.setdiag(0)
    a.eliminate_zeros()
    a.sum_duplicates()
    a.sort_indices()
    np.testing.assert_array_equal(off, a.indptr)
    np.testing.assert_array_equal(nb, a.indices)


def test_csr_build_duplicate_keeps_lowest_input_index(oracle):
    src = np.array([0, 1, 0, 0], dtype=np.int32)
    dst = np.array([1, 0, 1, 2], dtype=np.int32)
    w = np.array([10., 20., 30., 40.], dtype=np.float32)
    off, nb, wo = oracle.csr_build(src, dst, w, 3, oracle.SYMMETRIZE | oracle.DEDUPE)
    np.testing.assert_array_equal(off, [0, 2, 3, 4])
    np.testing.assert_array_equal(nb, [1, 2, 0, 0])
    # (0,1): inputs 0 (forward), 1 (reverse), 2 (forward) -> weight of input 0
    np.testing.assert_array_equal(wo, [10., 40., 10., 40.])


def test_csr_build_errors(oracle):
    e = np.zeros(0, dtype=np.int32)
    off, nb, _ = oracle.csr_build(e, e, None, 4, 7)
    np.testing.assert_array_equal(off, [0, 0, 0, 0, 0])
    assert nb.size == 0
    with pytest.raises(ValueError):
        oracle.csr_build(e, e, None, 4, 0, offset_bits=16)


# ----------------------------------------------------------------------------- alias
def _implied(prob, alias):
    """Exact probability of each outcome of an alias table (rationals)."""
    n = len(prob)
    out = [Fraction(0)] * n
    for i in range(n):
        pi = Fraction(float(prob[i]))
        out[i] += pi / n
        out[int(alias[i])] += (1 - pi) / n
    return out


def test_alias_hand_case(oracle):
    prob, alias = oracle.alias_build(np.array([0, 2], dtype=np.int32), [1.0, 3.0])
    np.testing.assert_array_equal(prob, [0.5, 1.0])
    np.testing.assert_array_equal(alias, [1, 1])


def test_alias_equal_weights(oracle):
    prob, alias = oracle.alias_build(np.array([0, 7], dtype=np.int64), [2.5] * 7)
    np.testing.assert_array_equal(prob, np.ones(7, dtype=np.float32))
    np.testing.assert_array_equal(alias, np.arange(7))


def test_alias_order_is_first_in_first_out(oracle):
    # weights 1,1,4,6 -> S=12, masses 4,4,16,24: small {0,1}, large {2,3}
    # (0 <- 2): mass2 = 16+4-12 = 8 -> small;  (1 <- 3): mass3 = 24+4-12 = 16 -> large
    # (2 <- 3): mass3 = 16+8-12 = 12 -> large (not < S); leftover 3: prob 1
    prob, alias = oracle.alias_build(np.array([0, 4], dtype=np.int32), [1., 1., 4., 6.])
    np.testing.assert_array_equal(alias, [2, 3, 3, 3])
    np.testing.assert_allclose(prob, [4 / 12, 4 / 12, 8 / 12, 1.0], rtol=1e-7)


def test_alias_zero_sum_and_single(oracle):
    prob, alias = oracle.alias_build(np.array([0, 3, 4, 4], dtype=np.int32), [0., 0., 0., 5.])
    np.testing.assert_array_equal(prob, [1, 1, 1, 1])
    np.testing.assert_array_equal(alias, [0, 1, 2, 0])


@pytest.mark.parametrize("seed", range(6))
def test_alias_implied_distribution_is_exact(oracle, seed):
    rng = np.random.default_rng(seed)
    sizes = rng.integers(1, 40, 30)
    seg = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    w = rng.lognormal(0, 1.5, seg[-1]).astype(np.float32)
    w[rng.random(w.size) < 0.15] = 0.0
    w[seg[3]:seg[4]] = 1.0                      # at least one segment is never all-zero
    prob, alias = oracle.alias_build(seg, w)
    assert prob.min() >= 0 and prob.max() <= 1
    for s in range(len(sizes)):
        lo, hi = seg[s], seg[s + 1]
        assert alias[lo:hi].min() >= 0 and alias[lo:hi].max() < hi - lo
        tot = sum(Fraction(float(x)) for x in w[lo:hi])
        if tot == 0:
            continue
        imp = _implied(prob[lo:hi], alias[lo:hi])
        assert sum(imp) == 1
        for j in range(hi - lo):
            want = Fraction(float(w[lo + j])) / tot
            # one fp32 rounding per prob entry, a few fp64 roundings of running masses
            assert abs(float(imp[j] - want)) <= 2.0 ** -23
            if w[lo + j] == 0:
                assert imp[j] == 0 or float(imp[j]) < 2.0 ** -40


def test_alias_draws_follow_the_weights(oracle):
    # sampled through the oracle's own negative sampler (slot + accept rule)
    w = np.array([5., 1., 0., 2., 8., 3., 1., 4.], dtype=np.float32)
    table = oracle.alias_build(np.array([0, 8], dtype=np.int32), w)
    draws = oracle.sample_negatives(table, 8, 200_000, 5, seed=99).ravel()
    counts = np.bincount(draws, minlength=8)
    assert counts[2] == 0
    keep = w > 0
    p = st.chisquare(counts[keep], counts.sum() * w[keep] / w.sum()).pvalue
    assert p > 0.01
