"""Parity at the full size of the benchmark workload (4M nodes, ~70M undirected
edges, node2vec walks of 80 nodes, 2,000,000-pair batches, dim 128), in the
launch shapes bench.py times.  Outputs too large to recompute on the CPU are
checked on samples the oracle computes one by one (walks by id, negatives by
pair index, pair blocks by walk) or through properties that hold at any size;
one whole SGNS batch is recomputed by the oracle and compared in full.
"""
import numpy as np
import pytest
import torch

from tolerances import assert_emb_close

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def gs():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2407_15452_amd import binding
    binding.lib()
    return binding


@pytest.fixture(scope="module")
def big(gs):
    from paper_2407_15452_amd import inputs
    wl = inputs.WORKLOADS[2]
    src, dst, _ = inputs.edge_list(wl, DEV)
    flags = gs.GS_SYMMETRIZE | gs.GS_DROP_SELF_LOOPS | gs.GS_DEDUPE
    g = gs.gs_csr_build(src, dst, None, wl.num_nodes, flags)
    torch.cuda.synchronize()
    off = g.offsets.cpu().numpy()
    nb = g.nbrs.cpu().numpy()
    return wl, g, off, nb, src, dst


def test_csr_properties_and_sampled_rows(gs, big):
    wl, g, off, nb, src, dst = big
    n = wl.num_nodes
    assert off[0] == 0 and off[-1] == nb.size and (np.diff(off) >= 0).all()
    # number of entries = 2 x distinct undirected edges of the input
    key = torch.minimum(src, dst).long() * n + torch.maximum(src, dst).long()
    assert nb.size == 2 * int(torch.unique(key).numel())
    # rows strictly ascending, no self loops, ids in range
    rows = np.repeat(np.arange(n, dtype=np.int64), np.diff(off))
    same_row = rows[1:] == rows[:-1]
    assert (nb[1:][same_row] > nb[:-1][same_row]).all()
    assert (nb != rows).all() and nb.min() >= 0 and nb.max() < n
    # sampled rows against the definition, straight from the edge list
    rng = np.random.default_rng(0)
    deg = np.diff(off)
    sample = np.concatenate([rng.integers(0, n, 40), np.argsort(deg)[-3:]])
    for v in sample:
        v = int(v)
        want = torch.unique(torch.cat([dst[src == v], src[dst == v]])).cpu().numpy()
        np.testing.assert_array_equal(nb[off[v]:off[v + 1]], want)
    # symmetry on a sample of entries: (a, b) present => (b, a) present
    for e in rng.integers(0, nb.size, 200):
        a, b = int(rows[e]), int(nb[e])
        r = nb[off[b]:off[b + 1]]
        i = np.searchsorted(r, a)
        assert i < r.size and r[i] == a


def test_node2vec_walks_sampled(gs, oracle, big):
    wl, g, off, nb, _, _ = big
    from paper_2407_15452_amd import inputs
    rng = np.random.default_rng(1)
    # the chunk shape bench.py walks for 20 batches, and one round over all nodes
    for first, count in ((4_000_123, 46_960), (0, 4_000_000)):
        starts = inputs.walk_starts(wl.num_nodes, first, count, DEV)
        walks = gs.gs_node2vec_walk(g, None, starts, wl.walk_len, wl.p, wl.q, wl.walk_seed,
                                    walk_id_base=first)
        pick = np.sort(rng.choice(count, 400, replace=False))
        got = walks[torch.as_tensor(pick, device=DEV)].cpu().numpy()
        st = starts[torch.as_tensor(pick, device=DEV)].cpu().numpy()
        for i, s, row in zip(pick, st, got):
            want = oracle.node2vec_walk(off, nb, np.array([s], dtype=np.int32), wl.walk_len,
                                        wl.p, wl.q, wl.walk_seed, walk_id_base=first + int(i))
            np.testing.assert_array_equal(row, want[0])
        # property over the whole launch: a walk from a node with edges never dies
        live = torch.as_tensor(np.diff(off) > 0, device=DEV)[starts.long()]
        assert bool((walks[live] >= 0).all())
        assert bool((walks[~live][:, 1:] == -1).all())
        del walks


def test_pairs_negatives_and_sgns_batch(gs, oracle, big):
    wl, g, off, nb, _, _ = big
    from paper_2407_15452_amd import inputs
    B, K, L, W = wl.batch_pairs, wl.num_neg, wl.walk_len, wl.window
    first, count = 0, 4000
    starts = inputs.walk_starts(wl.num_nodes, first, count, DEV)
    walks = gs.gs_node2vec_walk(g, None, starts, L, wl.p, wl.q, wl.walk_seed)
    centers, contexts, n_pairs = gs.gs_make_pairs(walks, W)
    h_walks = walks.cpu().numpy()
    lens = (h_walks >= 0).sum(1)
    per = np.where(lens > W, 2 * W * lens - W * (W + 1), lens * (lens - 1))
    assert n_pairs == per.sum() and n_pairs >= B
    base = np.concatenate([[0], np.cumsum(per)])
    rng = np.random.default_rng(2)
    hc, ho = centers.cpu().numpy(), contexts.cpu().numpy()
    for i in rng.choice(count, 60, replace=False):
        wc, wo = oracle.make_pairs(h_walks[i:i + 1], W)
        np.testing.assert_array_equal(hc[base[i]:base[i + 1]], wc)
        np.testing.assert_array_equal(ho[base[i]:base[i + 1]], wo)

    # negatives of one full batch, sampled by pair index
    noise_w = inputs.noise_weights(g.offsets)
    seg = torch.tensor([0, wl.num_nodes], dtype=torch.int64, device=DEV)
    noise = gs.gs_alias_build(seg, noise_w)
    pair_base = 37 * B
    negs = gs.gs_sample_negatives(noise, wl.num_nodes, B, K, wl.neg_seed, pair_index_base=pair_base)
    table = (noise.prob.cpu().numpy(), noise.alias.cpu().numpy())
    # the table itself against the oracle's construction (bit-exact, 4M entries)
    o_prob, o_alias = oracle.alias_build(np.array([0, wl.num_nodes], dtype=np.int64),
                                         noise_w.cpu().numpy())
    np.testing.assert_array_equal(table[1], o_alias)
    np.testing.assert_array_equal(table[0], o_prob)
    h_negs = negs.cpu().numpy()
    for i in rng.choice(B, 300, replace=False):
        want = oracle.sample_negatives(table, wl.num_nodes, 1, K, wl.neg_seed,
                                       pair_index_base=pair_base + int(i))
        np.testing.assert_array_equal(h_negs[i], want[0])
    assert h_negs.min() >= 0 and h_negs.max() < wl.num_nodes
    assert (np.diff(off)[h_negs.ravel()[:200_000]] > 0).all()     # never a zero-weight node

    # one whole 2,000,000-pair SGNS iteration against the oracle
    w_in, w_out = inputs.random_tables(wl.num_nodes, wl.dim, seed=5, scale=0.15, device=DEV)
    h_in, h_out = w_in.cpu().numpy(), w_out.cpu().numpy()
    c, o = centers[:B], contexts[:B]
    lr = 0.025
    loss = gs.gs_sgns_step(w_in, w_out, c, o, negs, lr)
    torch.cuda.synchronize()
    want = oracle.sgns_step(h_in, h_out, hc[:B], ho[:B], h_negs, lr)
    got = float(loss.item())
    assert abs(got - want) <= 1e-5 * abs(want)
    assert np.abs(w_in.cpu().numpy() - h_in).max() <= 1e-5
    assert np.abs(w_out.cpu().numpy() - h_out).max() <= 1e-5


def test_line_edges_full_size(gs, oracle, big):
    """2,000,000 LINE samples over the 140 M entries, uniform and weighted (alias table over
    all entries, built by the long-segment kernel), every sample against the oracle."""
    wl, g, off, nb, _, _ = big
    B = wl.batch_pairs
    base = (1 << 36) + 1
    c, o = gs.gs_sample_edges(g, None, B, seed=wl.walk_seed, sample_index_base=base)
    want_c, want_o = oracle.sample_edges(off, nb, B, seed=wl.walk_seed, sample_index_base=base)
    np.testing.assert_array_equal(c.cpu().numpy(), want_c)
    np.testing.assert_array_equal(o.cpu().numpy(), want_o)
    from paper_2407_15452_amd import inputs
    E = nb.size
    w = (inputs.hashed_u32(7, torch.arange(E, dtype=torch.int64, device=DEV), 3) >> 8).to(torch.float32)
    w = (w * (1.0 / (1 << 24))) ** 4 + 1e-3                         # skewed positive weights
    seg = torch.tensor([0, E], dtype=torch.int64, device=DEV)
    table = gs.gs_alias_build(seg, w, pack=True)
    c, o = gs.gs_sample_edges(g, table, B, seed=5)
    host_table = (table.prob.cpu().numpy(), table.alias.cpu().numpy())
    want_c, want_o = oracle.sample_edges(off, nb, B, seed=5, edge_alias=host_table)
    np.testing.assert_array_equal(c.cpu().numpy(), want_c)
    np.testing.assert_array_equal(o.cpu().numpy(), want_o)
    # the table itself on a property that holds at any size: implied mass of every entry
    # (own acceptance + what the aliases send to it) equals its weight share
    prob, alias = host_table
    mass = prob.astype(np.float64)
    np.add.at(mass, alias, 1.0 - prob.astype(np.float64))
    share = w.cpu().numpy().astype(np.float64)
    share *= E / share.sum()
    assert np.abs(mass - share).max() <= 1e-4 * max(1.0, share.max())


def test_storage_ops_full_size(gs, oracle, big):
    """The ids of one 2,000,000-pair batch (14 M ids): merged ids against numpy, get and put
    of the distinct rows against the oracle on a sample of rows."""
    wl, g, off, nb, _, _ = big
    from paper_2407_15452_amd import inputs
    n, d, B, K = wl.num_nodes, wl.dim, wl.batch_pairs, wl.num_neg
    c, o = gs.gs_sample_edges(g, None, B, seed=3)
    negs = gs.gs_sample_negatives(None, n, B, K, seed=4, device=DEV)
    ids = torch.cat([c, o, negs.reshape(-1)])
    u, count, inv = gs.gs_unique_ids(ids, n)
    k = int(count.item())
    want_u, want_inv = np.unique(ids.cpu().numpy(), return_inverse=True)
    assert k == want_u.size
    np.testing.assert_array_equal(u[:k].cpu().numpy(), want_u)
    np.testing.assert_array_equal(inv.cpu().numpy(), want_inv)
    table = inputs.random_tables(n, d, seed=6, scale=0.2, device=DEV)[0]
    before = table.clone()
    block = gs.gs_get_rows(table, u, count=count)
    assert torch.equal(block[:k], before[u[:k].long()])
    delta = inputs.random_tables(k, d, seed=8, scale=1.0, device=DEV)[1]
    gs.gs_put_rows(table, u, delta, -0.125, count=count)
    rng = np.random.default_rng(0)
    pick = np.sort(rng.choice(k, 2000, replace=False))
    rows = want_u[pick]
    sub = before[torch.as_tensor(rows, device=DEV).long()].cpu().numpy().copy()
    oracle.put_rows(sub, np.arange(rows.size, dtype=np.int32), delta.cpu().numpy()[pick], -0.125)
    np.testing.assert_array_equal(table[torch.as_tensor(rows, device=DEV).long()].cpu().numpy(), sub)
    untouched = torch.ones(n, dtype=torch.bool, device=DEV)
    untouched[u[:k].long()] = False
    assert torch.equal(table[untouched], before[untouched])


def test_line_first_order_and_optimizer_steps_full_batch(gs, oracle, big):
    """At the full batch size of the benchmark (2,000,000 pairs over 4 M rows of 128 floats), each
    recomputed whole by the oracle: a first-order LINE iteration on sorted sampled edges, a
    momentum iteration and an Adam iteration on the same batch."""
    wl, g, off, nb, _, _ = big
    from paper_2407_15452_amd import inputs
    n, d, B, K = wl.num_nodes, wl.dim, wl.batch_pairs, wl.num_neg
    c_raw, o_raw = gs.gs_sample_edges(g, None, B, seed=61)
    c, o = gs.gs_sort_pairs(c_raw, o_raw, n)
    want_c, want_o = oracle.sort_pairs(c_raw.cpu().numpy(), o_raw.cpu().numpy(), n)
    np.testing.assert_array_equal(c.cpu().numpy(), want_c)
    np.testing.assert_array_equal(o.cpu().numpy(), want_o)
    negs = gs.gs_sample_negatives(None, n, B, K, seed=62, device=DEV)
    hc, ho, hn = c.cpu().numpy(), o.cpu().numpy(), negs.cpu().numpy()

    w = inputs.random_tables(n, d, seed=7, scale=0.15, device=DEV)[0]
    h_w = w.cpu().numpy()
    loss = gs.gs_line1_step(w, c, o, negs, 0.025)
    want = oracle.line1_step(h_w, hc, ho, hn, 0.025)
    assert abs(float(loss.item()) - want) <= 1e-5 * abs(want)
    assert np.abs(w.cpu().numpy() - h_w).max() <= 1e-5
    del w, h_w

    tabs = list(inputs.random_tables(n, d, seed=8, scale=0.15, device=DEV))
    tabs += list(inputs.random_tables(n, d, seed=9, scale=0.01, device=DEV))
    host = [t.cpu().numpy() for t in tabs]
    loss = gs.gs_sgns_momentum_step(*tabs, c, o, negs, 0.025, 0.9)
    want = oracle.sgns_momentum_step(*host, hc, ho, hn, 0.025, 0.9)
    assert abs(float(loss.item()) - want) <= 1e-5 * abs(want)
    for t, h in zip(tabs, host):
        assert_emb_close(t.cpu().numpy(), h)

    # Adam, first iteration (moments from zero), on the model the momentum step left (the
    # oracle's copy on both sides)
    for t, h in zip(tabs[:2], host[:2]):
        t.copy_(torch.from_numpy(h))
    tabs = tabs[:2] + [torch.zeros_like(tabs[0]) for _ in range(4)]
    host = host[:2] + [np.zeros_like(host[0]) for _ in range(4)]
    before = [h.copy() for h in host[:2]]
    loss = gs.gs_sgns_adam_step(*tabs, c, o, negs, 0.01, 0.9, 0.999, 1e-8, 1)
    want = oracle.sgns_adam_step(*host, hc, ho, hn, 0.01, 0.9, 0.999, 1e-8, 1)
    assert abs(float(loss.item()) - want) <= 1e-5 * abs(want)
    got = [t.cpu().numpy() for t in tabs]
    for which in (2, 3, 4, 5):
        assert (np.abs(got[which] - host[which]) <= 1e-6 + 1e-5 * np.abs(host[which])).all()
    step = np.float64(np.float32(0.01)) / (1.0 - np.float64(np.float32(0.9)))
    root = np.sqrt(1.0 - np.float64(np.float32(0.999)))
    for which in (0, 1):
        safe = (np.sqrt(host[which + 4].astype(np.float64)) / root + 1e-8) >= 1e-3
        assert np.abs(got[which] - host[which])[safe].max() <= 1e-5
        assert np.abs(got[which] - host[which]).max() <= 2.0 * step + 1e-5
        m, v = got[which + 2].astype(np.float64), got[which + 4].astype(np.float64)
        expect = before[which] - step * m / (np.sqrt(v) / root + np.float64(np.float32(1e-8)))
        assert np.abs(got[which] - expect).max() <= 1e-6


def test_workload1_full_size(gs, oracle):
    """Workload 1 at its own shape (1 M nodes, 10 M undirected edges, uniform walks of 40
    nodes, window 5, K = 5, dim 128 fp32, 1,048,576-pair batches): the CSR and the noise table
    against the oracle in full, a 4 M-walk launch sampled by walk id, pair blocks by walk,
    negatives by pair index, and one whole batch recomputed by the oracle."""
    from paper_2407_15452_amd import inputs
    wl = inputs.WORKLOADS[1]
    N, B, K, L, W = wl.num_nodes, wl.batch_pairs, wl.num_neg, wl.walk_len, wl.window
    rng = np.random.default_rng(11)
    src, dst, _ = inputs.edge_list(wl, DEV)
    flags = gs.GS_SYMMETRIZE | gs.GS_DROP_SELF_LOOPS | gs.GS_DEDUPE
    g = gs.gs_csr_build(src, dst, None, N, flags)
    torch.cuda.synchronize()
    off, nb = g.offsets.cpu().numpy(), g.nbrs.cpu().numpy()
    want_off, want_nb, _ = oracle.csr_build(src.cpu().numpy(), dst.cpu().numpy(), None, N, flags)
    np.testing.assert_array_equal(off, want_off)
    np.testing.assert_array_equal(nb, want_nb)
    del src, dst

    noise_w = inputs.noise_weights(g.offsets)
    seg = torch.tensor([0, N], dtype=torch.int64, device=DEV)
    noise = gs.gs_alias_build(seg, noise_w)
    o_prob, o_alias = oracle.alias_build(np.array([0, N], dtype=np.int64), noise_w.cpu().numpy())
    np.testing.assert_array_equal(noise.alias.cpu().numpy(), o_alias)
    np.testing.assert_array_equal(noise.prob.cpu().numpy(), o_prob)

    # the stand-alone launch bench.py times (4 M walks), sampled by walk id
    first, count = 3_000_017, 4_000_000
    starts = inputs.walk_starts(N, first, count, DEV)
    walks = gs.gs_random_walk(g, None, starts, L, wl.walk_seed, walk_id_base=first)
    pick = np.sort(rng.choice(count, 400, replace=False))
    got = walks[torch.as_tensor(pick, device=DEV)].cpu().numpy()
    st = starts[torch.as_tensor(pick, device=DEV)].cpu().numpy()
    for i, s, row in zip(pick, st, got):
        want = oracle.random_walk(off, nb, np.array([s], dtype=np.int32), L, wl.walk_seed,
                                  walk_id_base=first + int(i))
        np.testing.assert_array_equal(row, want[0])
    live = torch.as_tensor(np.diff(off) > 0, device=DEV)[starts.long()]
    assert bool((walks[live] >= 0).all()) and bool((walks[~live][:, 1:] == -1).all())
    del walks

    # a chunk of walks that holds more than one batch, whole against the oracle
    count = 6000
    starts = inputs.walk_starts(N, 0, count, DEV)
    walks = gs.gs_random_walk(g, None, starts, L, wl.walk_seed)
    h_walks = oracle.random_walk(off, nb, starts.cpu().numpy(), L, wl.walk_seed)
    np.testing.assert_array_equal(walks.cpu().numpy(), h_walks)
    centers, contexts, n_pairs = gs.gs_make_pairs(walks, W)
    hc, ho = oracle.make_pairs(h_walks, W)
    assert n_pairs == hc.size and n_pairs >= B
    np.testing.assert_array_equal(centers[:n_pairs].cpu().numpy(), hc)
    np.testing.assert_array_equal(contexts[:n_pairs].cpu().numpy(), ho)

    pair_base = 5 * B
    negs = gs.gs_sample_negatives(noise, N, B, K, wl.neg_seed, pair_index_base=pair_base)
    h_negs = oracle.sample_negatives((o_prob, o_alias), N, B, K, wl.neg_seed, pair_index_base=pair_base)
    np.testing.assert_array_equal(negs.cpu().numpy(), h_negs)

    # one whole 1,048,576-pair iteration
    w_in, w_out = inputs.random_tables(N, wl.dim, seed=15, scale=0.15, device=DEV)
    h_in, h_out = w_in.cpu().numpy(), w_out.cpu().numpy()
    lr = 0.025
    loss = gs.gs_sgns_step(w_in, w_out, centers[:B], contexts[:B], negs, lr)
    torch.cuda.synchronize()
    want = oracle.sgns_step(h_in, h_out, hc[:B], ho[:B], h_negs, lr)
    assert abs(float(loss.item()) - want) <= 1e-5 * abs(want)
    assert np.abs(w_in.cpu().numpy() - h_in).max() <= 1e-5
    assert np.abs(w_out.cpu().numpy() - h_out).max() <= 1e-5
