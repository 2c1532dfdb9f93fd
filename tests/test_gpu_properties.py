"""Randomised small cases (hypothesis), library against oracle through the C boundary:
odd shapes, ragged tails, empty rows, dead ends, tiny batches."""
import numpy as np
import pytest
import torch
from hypothesis import HealthCheck, given, settings, strategies as st

from tolerances import assert_emb_close, assert_half_close

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
COMMON = dict(deadline=None, derandomize=True, suppress_health_check=[HealthCheck.function_scoped_fixture,
                                                    HealthCheck.too_slow])


@pytest.fixture(scope="module")
def gs():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2407_15452_amd import binding
    binding.lib()
    return binding


def _t(a):
    return torch.as_tensor(np.ascontiguousarray(a)).to(DEV)


def _graph(rng, n, m, oracle, directed):
    src = rng.integers(-1, n + 1, m).astype(np.int32)          # a few ids out of range
    dst = rng.integers(-1, n + 1, m).astype(np.int32)
    flags = oracle.DROP_SELF_LOOPS | oracle.DEDUPE | (0 if directed else oracle.SYMMETRIZE)
    return src, dst, flags


@settings(max_examples=40, **COMMON)
@given(st.integers(1, 60), st.integers(0, 300), st.integers(0, 7), st.sampled_from([32, 64]),
       st.booleans(), st.integers(0, 2 ** 31 - 1))
def test_csr_build_random(gs, oracle, n, m, flags, bits, weighted, seed):
    rng = np.random.default_rng(seed)
    src = rng.integers(-1, n + 1, m).astype(np.int32)
    dst = rng.integers(-1, n + 1, m).astype(np.int32)
    w = rng.random(m).astype(np.float32) if weighted else None
    off, nb, ww = oracle.csr_build(src, dst, w, n, flags, offset_bits=bits)
    g = gs.gs_csr_build(_t(src), _t(dst), None if w is None else _t(w), n, flags, offset_bits=bits)
    np.testing.assert_array_equal(g.offsets.cpu().numpy(), off)
    np.testing.assert_array_equal(g.nbrs.cpu().numpy()[:nb.size], nb)
    if weighted:
        np.testing.assert_array_equal(g.weights.cpu().numpy()[:nb.size], ww)


@settings(max_examples=40, **COMMON)
@given(st.integers(2, 80), st.integers(1, 400), st.integers(1, 40), st.booleans(), st.booleans(),
       st.sampled_from([(1.0, 1.0), (0.5, 2.0), (4.0, 0.25), (0.25, 0.5)]), st.integers(0, 2 ** 31 - 1))
def test_walks_random(gs, oracle, n, m, walk_len, directed, weighted, pq, seed):
    rng = np.random.default_rng(seed)
    src, dst, flags = _graph(rng, n, m, oracle, directed)
    w = rng.lognormal(0, 1, m).astype(np.float32) if weighted else None
    off, nb, ww = oracle.csr_build(src, dst, w, n, flags)
    g = gs.gs_csr_build(_t(src), _t(dst), None if w is None else _t(w), n, flags)
    table_h = table_d = None
    if weighted and nb.size:
        table_h = oracle.alias_build(off, ww)
        table_d = gs.gs_alias_build(g.offsets, g.weights[:nb.size].contiguous())
        np.testing.assert_array_equal(table_d.prob.cpu().numpy(), table_h[0])
        np.testing.assert_array_equal(table_d.alias.cpu().numpy(), table_h[1])
    starts = rng.integers(-1, n + 1, 150).astype(np.int32)       # some starts are not nodes
    base = int(rng.integers(0, 1 << 40))
    want = oracle.random_walk(off, nb, starts, walk_len, seed, alias=table_h, walk_id_base=base)
    got = gs.gs_random_walk(g, table_d, _t(starts), walk_len, seed, walk_id_base=base)
    np.testing.assert_array_equal(got.cpu().numpy(), want)
    p, q = pq
    want = oracle.node2vec_walk(off, nb, starts, walk_len, p, q, seed, alias=table_h, walk_id_base=base)
    got = gs.gs_node2vec_walk(g, table_d, _t(starts), walk_len, p, q, seed, walk_id_base=base)
    np.testing.assert_array_equal(got.cpu().numpy(), want)


@settings(max_examples=40, **COMMON)
@given(st.integers(1, 70), st.integers(1, 12), st.integers(0, 200), st.integers(0, 2 ** 31 - 1))
def test_make_pairs_random(gs, oracle, walk_len, window, num_walks, seed):
    rng = np.random.default_rng(seed)
    walks = rng.integers(0, 1000, (num_walks, walk_len)).astype(np.int32)
    for i in range(num_walks):
        if rng.random() < 0.4:
            walks[i, rng.integers(0, walk_len + 1):] = -1
    wc, wo = oracle.make_pairs(walks, window)
    c, o, n = gs.gs_make_pairs(_t(walks).reshape(num_walks, walk_len), window)
    assert n == wc.size
    np.testing.assert_array_equal(c.cpu().numpy(), wc)
    np.testing.assert_array_equal(o.cpu().numpy(), wo)


@settings(max_examples=40, **COMMON)
@given(st.sampled_from([4, 8, 12, 64, 100, 128, 192]), st.integers(0, 9), st.integers(1, 400),
       st.integers(1, 300), st.sampled_from(["f32", "bf16", "f16"]), st.integers(0, 2 ** 31 - 1))
def test_sgns_step_random(gs, oracle, dim, k, b, n, fmt, seed):
    if fmt != "f32":
        dim = max(8, dim // 8 * 8)
    rng = np.random.default_rng(seed)
    tdt, code = {"f32": (torch.float32, oracle.F32), "bf16": (torch.bfloat16, oracle.BF16),
                 "f16": (torch.float16, oracle.F16)}[fmt]
    w_in = torch.tensor(rng.normal(0, 0.3, (n, dim)), dtype=torch.float32).to(tdt)
    w_out = torch.tensor(rng.normal(0, 0.3, (n, dim)), dtype=torch.float32).to(tdt)
    c = rng.integers(0, n, b).astype(np.int32)
    o = rng.integers(0, n, b).astype(np.int32)
    neg = rng.integers(0, n, (b, k)).astype(np.int32)
    bits = lambda t: (t.numpy().copy() if fmt == "f32"  # noqa: E731
                      else t.view(torch.int16).numpy().view(np.uint16).copy())
    h_in, h_out = bits(w_in), bits(w_out)
    want = oracle.sgns_step(h_in, h_out, c, o, neg, 0.05, dtype=code)
    d_in, d_out = w_in.to(DEV), w_out.to(DEV)
    loss = gs.gs_sgns_step(d_in, d_out, _t(c), _t(o), _t(neg).reshape(b, k), 0.05)
    assert abs(float(loss.item()) - want) <= 1e-5 * abs(want) + 1e-12
    for d_t, h_t in ((d_in, h_in), (d_out, h_out)):
        got = bits(d_t.cpu())
        if fmt == "f32":
            assert_emb_close(got, h_t)
        else:
            # tiny tables: one element that rounds the other way is already a large fraction
            assert_half_close(got, h_t, fmt, flip_fraction=1.0)


@settings(max_examples=40, **COMMON)
@given(st.lists(st.integers(-3, 5000), max_size=400), st.integers(1, 4000))
def test_unique_and_sort_random(gs, oracle, ids, num_nodes):
    ids = np.array(ids, dtype=np.int32)
    u, count, inv = gs.gs_unique_ids(_t(ids).reshape(-1), num_nodes)
    want_u, want_inv = oracle.unique_ids(ids, num_nodes)
    k = int(count.item())
    assert k == want_u.size
    np.testing.assert_array_equal(u[:k].cpu().numpy(), want_u)
    np.testing.assert_array_equal(inv.cpu().numpy(), want_inv)
    other = (ids.astype(np.int64) * 7919 % 1000).astype(np.int32)
    sc, so = gs.gs_sort_pairs(_t(ids).reshape(-1), _t(other).reshape(-1), num_nodes)
    wc, wo = oracle.sort_pairs(ids, other, num_nodes)
    np.testing.assert_array_equal(sc.cpu().numpy(), wc)
    np.testing.assert_array_equal(so.cpu().numpy(), wo)
