"""GPU parity for the LINE path: gs_sample_edges against the oracle (bit-exact),
then LINE batches (sampled edges + negatives + the SGNS step) against the oracle
to the SGNS tolerances."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
from tolerances import EMB_ATOL, LOSS_RTOL, assert_half_close  # noqa: E402


@pytest.fixture(scope="module")
def gs():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2407_15452_amd import binding
    binding.lib()          # raises if libgs.so was not built
    return binding


def _t(a, dtype=None):
    t = torch.as_tensor(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(DEV)


@pytest.fixture(scope="module")
def graph0(gs, oracle):
    from paper_2407_15452_amd import inputs
    wl = inputs.WORKLOADS[0]
    src, dst, _ = inputs.edge_list(wl, "cpu")
    flags = oracle.SYMMETRIZE | oracle.DROP_SELF_LOOPS | oracle.DEDUPE
    off, nb, _ = oracle.csr_build(src.numpy(), dst.numpy(), None, wl.num_nodes, flags)
    g = gs.gs_csr_build(src.to(DEV), dst.to(DEV), None, wl.num_nodes, flags)
    torch.cuda.synchronize()
    return wl, (off, nb), g


@pytest.mark.parametrize("count,base", [(0, 0), (1, 0), (255, 7), (100_003, (1 << 33) + 5)])
def test_sample_edges_uniform(gs, oracle, graph0, count, base):
    wl, (off, nb), g = graph0
    want_c, want_o = oracle.sample_edges(off, nb, count, seed=77, sample_index_base=base)
    c, o = gs.gs_sample_edges(g, None, count, seed=77, sample_index_base=base)
    np.testing.assert_array_equal(c.cpu().numpy(), want_c)
    np.testing.assert_array_equal(o.cpu().numpy(), want_o)


@pytest.mark.parametrize("pack", [False, True])
def test_sample_edges_weighted(gs, oracle, graph0, pack):
    wl, (off, nb), g = graph0
    rng = np.random.default_rng(3)
    w = rng.lognormal(0, 1.5, nb.size).astype(np.float32)
    w[rng.random(nb.size) < 0.1] = 0
    seg = np.array([0, nb.size], dtype=np.int64)
    table = oracle.alias_build(seg, w)
    a = gs.gs_alias_build(_t(seg), _t(w), pack=pack)
    assert (a.packed is not None) == pack
    np.testing.assert_array_equal(a.prob.cpu().numpy(), table[0])
    want_c, want_o = oracle.sample_edges(off, nb, 200_001, seed=5, edge_alias=table)
    c, o = gs.gs_sample_edges(g, a, 200_001, seed=5)
    np.testing.assert_array_equal(c.cpu().numpy(), want_c)
    np.testing.assert_array_equal(o.cpu().numpy(), want_o)
    # entries of weight zero are never drawn
    src = np.repeat(np.arange(wl.num_nodes), np.diff(off))
    dead = set(zip(src[w == 0].tolist(), nb[w == 0].tolist()))
    assert not dead & set(zip(want_c.tolist(), want_o.tolist()))


def test_sample_edges_int64_offsets_and_empty_rows(gs, oracle):
    rng = np.random.default_rng(1)
    n, m = 5_000, 20_000
    src = (rng.integers(0, n // 3, m) * 3).astype(np.int32)        # two of three rows stay empty
    dst = rng.integers(0, n, m).astype(np.int32)
    flags = oracle.DROP_SELF_LOOPS | oracle.DEDUPE
    off, nb, _ = oracle.csr_build(src, dst, None, n, flags, offset_bits=64)
    g = gs.gs_csr_build(_t(src), _t(dst), None, n, flags, offset_bits=64)
    assert g.offsets.dtype == torch.int64
    want_c, want_o = oracle.sample_edges(off, nb, 50_000, seed=9)
    c, o = gs.gs_sample_edges(g, None, 50_000, seed=9)
    np.testing.assert_array_equal(c.cpu().numpy(), want_c)
    np.testing.assert_array_equal(o.cpu().numpy(), want_o)
    assert (want_c % 3 == 0).all()
    # last row non-empty / first rows empty
    off2, nb2, _ = oracle.csr_build([7, 7], [0, 3], None, 8, 0)
    g2 = gs.gs_csr_build(_t(np.array([7, 7], dtype=np.int32)), _t(np.array([0, 3], dtype=np.int32)),
                         None, 8, 0)
    c, o = gs.gs_sample_edges(g2, None, 100, seed=1)
    want_c, want_o = oracle.sample_edges(off2, nb2, 100, seed=1)
    np.testing.assert_array_equal(c.cpu().numpy(), want_c)
    np.testing.assert_array_equal(o.cpu().numpy(), want_o)
    assert (want_c == 7).all()


def test_sample_edges_argument_errors(gs, graph0):
    wl, _, g = graph0
    empty = gs.Csr(torch.zeros(5, dtype=torch.int32, device=DEV),
                   torch.zeros(0, dtype=torch.int32, device=DEV))
    with pytest.raises(gs.GsError):
        gs.gs_sample_edges(empty, None, 10, seed=1)
    with pytest.raises(gs.GsError):
        gs.gs_sample_edges(g, None, -1, seed=1)


def test_line_batches_workload0(gs, oracle, graph0):
    """Ten LINE iterations (second-order proximity): B sampled edges, K negatives per
    source node from degree^0.75, one SGNS step each; compared step by step."""
    from paper_2407_15452_amd import inputs
    wl, (off, nb), g = graph0
    n, d, K, B = wl.num_nodes, wl.dim, 5, 16_384
    nw = inputs.noise_weights(torch.as_tensor(off)).numpy()
    seg = np.array([0, n], dtype=np.int32)
    noise_h = oracle.alias_build(seg, nw)
    noise_d = gs.gs_alias_build(_t(seg), _t(nw))
    w_in, w_out = inputs.random_tables(n, d, 12, 0.3)
    h_in, h_out = w_in.numpy().copy(), w_out.numpy().copy()
    d_in, d_out = w_in.to(DEV), w_out.to(DEV)
    lr = 0.025
    first = last = None
    for it in range(10):
        hc, ho = oracle.sample_edges(off, nb, B, seed=31, sample_index_base=it * B)
        hn = oracle.sample_negatives(noise_h, n, B, K, seed=32, pair_index_base=it * B)
        c, o = gs.gs_sample_edges(g, None, B, seed=31, sample_index_base=it * B)
        neg = gs.gs_sample_negatives(noise_d, n, B, K, seed=32, pair_index_base=it * B)
        np.testing.assert_array_equal(c.cpu().numpy(), hc)
        np.testing.assert_array_equal(neg.cpu().numpy(), hn)
        loss = gs.gs_sgns_step(d_in, d_out, c, o, neg, lr)
        want = oracle.sgns_step(h_in, h_out, hc, ho, hn, lr)
        got = float(loss.item())
        assert abs(got - want) <= LOSS_RTOL * abs(want)
        first = want if first is None else first
        last = want
        assert np.abs(d_in.cpu().numpy() - h_in).max() <= EMB_ATOL * (it + 1)
        assert np.abs(d_out.cpu().numpy() - h_out).max() <= EMB_ATOL * (it + 1)
    assert last < first          # the objective goes down


def _bf16_bits(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("dim,k,b,dtype", [(128, 5, 50_001, "f32"), (64, 3, 7_777, "f32"),
                                           (8, 0, 300, "f32"), (256, 10, 9_999, "bf16")])
def test_line1_step(gs, oracle, dim, k, b, dtype):
    """First-order LINE (one table on both sides): two consecutive iterations on batches in which
    sources also appear as targets and negatives (the reads must still see the old rows)."""
    from paper_2407_15452_amd import inputs
    n = 3000
    table = inputs.random_tables(n, dim, seed=dim + k, scale=2.0 / dim ** 0.5)[0]
    rng = np.random.default_rng(b)
    if dtype == "bf16":
        d_w = table.to(torch.bfloat16).to(DEV)
        h_w = _bf16_bits(d_w).copy()
        code = oracle.BF16
    else:
        d_w = table.to(DEV)
        h_w = table.numpy().copy()
        code = oracle.F32
    for it in range(2):
        s = (n * rng.random(b) ** 2).astype(np.int32)                 # hubs are sources often
        t = rng.integers(0, n, b).astype(np.int32)
        t[::7] = s[::7]                                               # self pairs
        neg = (n * rng.random((b, k)) ** 3).astype(np.int32)
        want = oracle.line1_step(h_w, s, t, neg, 0.01, dtype=code)
        loss = gs.gs_line1_step(d_w, _t(s), _t(t), _t(neg), 0.01)
        torch.cuda.synchronize()
        assert abs(float(loss.item()) - want) <= LOSS_RTOL * abs(want)
        if dtype == "bf16":
            # two roundings per element: a flip in the first moves the second by one step
            assert_half_close(_bf16_bits(d_w), h_w, "bf16", steps=2)
            d_w.copy_(torch.from_numpy(h_w.view(np.int16)).view(torch.bfloat16))
        else:
            assert np.abs(d_w.cpu().numpy() - h_w).max() <= EMB_ATOL


def test_line1_training_on_workload0(gs, oracle, graph0):
    """Ten first-order LINE iterations on sampled edges of workload 0, checked step by step."""
    from paper_2407_15452_amd import inputs
    wl, (off, nb), g = graph0
    n, d, K, B = wl.num_nodes, wl.dim, 5, 16_384
    table = inputs.random_tables(n, d, 21, 0.3)[0]
    h_w, d_w = table.numpy().copy(), table.to(DEV)
    first = last = None
    for it in range(10):
        c, o = gs.gs_sample_edges(g, None, B, seed=41, sample_index_base=it * B)
        neg = gs.gs_sample_negatives(None, n, B, K, seed=42, pair_index_base=it * B, device=DEV)
        loss = gs.gs_line1_step(d_w, c, o, neg, 0.025)
        want = oracle.line1_step(h_w, c.cpu().numpy(), o.cpu().numpy(), neg.cpu().numpy(), 0.025)
        assert abs(float(loss.item()) - want) <= LOSS_RTOL * abs(want)
        assert np.abs(d_w.cpu().numpy() - h_w).max() <= EMB_ATOL * (it + 1)
        first = want if first is None else first
        last = want
    assert last < first


def test_line1_step_argument_errors(gs):
    w = torch.zeros((10, 8), dtype=torch.float32, device=DEV)
    i = torch.zeros(4, dtype=torch.int32, device=DEV)
    n = torch.zeros((4, 2), dtype=torch.int32, device=DEV)
    small = torch.empty(256, dtype=torch.uint8, device=DEV)
    with pytest.raises(gs.GsError):
        gs.gs_line1_step(w, i, i, n, 0.1, ws=small)
    bad = i.clone(); bad[1] = 10
    assert np.isnan(float(gs.gs_line1_step(w, bad, i, n, 0.1).item()))


@pytest.mark.parametrize("n,num_nodes", [(0, 10), (1, 10), (4097, 300), (200_003, 1_000_000),
                                         (50_000, (1 << 31) - 1)])
def test_sort_pairs(gs, oracle, n, num_nodes):
    rng = np.random.default_rng(n + 1)
    c = rng.integers(0, min(num_nodes, 1 << 22), n).astype(np.int32)
    o = rng.integers(0, 1 << 30, n).astype(np.int32)
    if n > 100:
        c[::97] = -3                                          # not rows: go last
        if num_nodes < (1 << 31) - 1:
            c[5::101] = num_nodes
    want_c, want_o = oracle.sort_pairs(c, o, num_nodes)
    got_c, got_o = gs.gs_sort_pairs(_t(c).reshape(-1), _t(o).reshape(-1), num_nodes)
    np.testing.assert_array_equal(got_c.cpu().numpy(), want_c)
    np.testing.assert_array_equal(got_o.cpu().numpy(), want_o)


def test_sorted_line_batch_gives_the_same_step(gs, oracle, graph0):
    """A LINE batch reordered by source id: the step's result is that of the unsorted batch
    with the negatives permuted alike (sums over the batch), within the step's tolerance."""
    from paper_2407_15452_amd import inputs
    wl, (off, nb), g = graph0
    n, d, K, B = wl.num_nodes, wl.dim, 5, 30_000
    c, o = gs.gs_sample_edges(g, None, B, seed=51)
    sc, so = gs.gs_sort_pairs(c, o, n)
    assert bool((sc[1:] >= sc[:-1]).all())
    neg = gs.gs_sample_negatives(None, n, B, K, seed=52, device=DEV)
    w_in, w_out = inputs.random_tables(n, d, 3, 0.3)
    d_in, d_out = w_in.to(DEV), w_out.to(DEV)
    loss = gs.gs_sgns_step(d_in, d_out, sc, so, neg, 0.02)
    h_in, h_out = w_in.numpy().copy(), w_out.numpy().copy()
    want = oracle.sgns_step(h_in, h_out, sc.cpu().numpy(), so.cpu().numpy(), neg.cpu().numpy(), 0.02)
    assert abs(float(loss.item()) - want) <= LOSS_RTOL * abs(want)
    assert np.abs(d_in.cpu().numpy() - h_in).max() <= EMB_ATOL
    assert np.abs(d_out.cpu().numpy() - h_out).max() <= EMB_ATOL
    with pytest.raises(gs.GsError):
        gs.gs_sort_pairs(c, o, n, centers_out=c, contexts_out=o)
