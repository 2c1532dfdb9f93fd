"""Parity at the full size of the two largest workloads, on one GPU:

  workload 3  weighted bipartite graph, 25M nodes, ~970M CSR entries, per-row
              alias tables, weighted walks, K = 10, dim 256 bf16 tables
  workload 4  directed R-MAT, 100M nodes, ~1.6G CSR entries, 64-bit offsets,
              dim 128 fp32 tables (2 x 51 GB resident)

Nothing of this size can be recomputed whole on the CPU, so the oracle checks
samples it can compute one by one: CSR rows from the edge list, per-row alias
tables, walks by id, pair blocks by walk, negatives by pair index, and -- for
one SGNS iteration at the full batch size -- individual destination rows and
centre rows, each recomputed by the oracle from exactly the terms of the batch
that touch it (an iteration touches no other row).  The batch loss is
recomputed by the oracle over the whole batch, in chunks on compacted tables.
"""
import numpy as np
import pytest
import torch

from tolerances import HALF_FLIP_FRACTION, emb_bound

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def gs():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    if torch.cuda.get_device_properties(0).total_memory < 250e9:
        pytest.skip("needs the 288 GB of an MI355X")
    from paper_2407_15452_amd import binding
    binding.lib()
    return binding


def _bits(t):
    """Host copy of table rows in the oracle's storage type."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16).copy()
    return t.cpu().numpy().copy()


def _rows(table, ids):
    return _bits(table[torch.as_tensor(ids, dtype=torch.long, device=table.device)])


def _check_rows(got, want, dtype, tally):
    """fp32: 1e-5 max-abs.  bf16: every element within one bf16 step (or the fp32 bound where
    the sum cancels); the number of elements that are not bit-identical is tallied for the caller."""
    if dtype == "bf16":
        near = np.abs(got.astype(np.int32) - want.astype(np.int32)) <= 1
        gv = (got.astype(np.uint32) << 16).view(np.float32)
        wv = (want.astype(np.uint32) << 16).view(np.float32)
        assert bool((near | (np.abs(gv - wv) <= emb_bound(wv))).all())
        tally[0] += int((got != want).sum())
        tally[1] += got.size
    else:
        assert float(np.abs(got - want).max()) <= 1e-5


def _run_workload(gs, oracle, index, num_walks):
    from paper_2407_15452_amd import inputs
    wl = inputs.WORKLOADS[index]
    odt = oracle.BF16 if wl.dtype == "bf16" else oracle.F32
    rng = np.random.default_rng(index)
    N, B, K, L, W = wl.num_nodes, wl.batch_pairs, wl.num_neg, wl.walk_len, wl.window

    # ---- CSR ------------------------------------------------------------------------------
    src, dst, w = inputs.edge_list(wl, DEV)
    flags = gs.GS_DROP_SELF_LOOPS | gs.GS_DEDUPE | (0 if wl.directed else gs.GS_SYMMETRIZE)
    g = gs.gs_csr_build(src, dst, w, N, flags, wl.offset_bits)
    torch.cuda.synchronize()
    off = g.offsets.cpu().numpy()
    nb = g.nbrs.cpu().numpy()
    assert off.dtype == (np.int64 if wl.offset_bits == 64 else np.int32)
    assert off[0] == 0 and off[-1] == nb.size and (np.diff(off) >= 0).all()
    deg = np.diff(off)
    sample_nodes = np.concatenate([rng.integers(0, N, 30), np.argsort(deg)[-2:]])
    for v in sample_nodes:
        v = int(v)
        if wl.directed:
            want = torch.unique(dst[(src == v) & (dst != v)])
        else:
            want = torch.unique(torch.cat([dst[src == v], src[dst == v]]))
            want = want[want != v]
        np.testing.assert_array_equal(nb[off[v]:off[v + 1]], want.cpu().numpy())
    del src, dst
    torch.cuda.empty_cache()

    # ---- alias tables ---------------------------------------------------------------------
    row_alias = table = None
    if wl.weighted:
        row_alias = gs.gs_alias_build(g.offsets, g.weights)
        prob, alias = row_alias.prob.cpu().numpy(), row_alias.alias.cpu().numpy()
        hw = g.weights.cpu().numpy()
        for v in sample_nodes:
            lo, hi = int(off[v]), int(off[v + 1])
            if hi == lo:
                continue
            p, a = oracle.alias_build(np.array([0, hi - lo], dtype=np.int64), hw[lo:hi])
            np.testing.assert_array_equal(prob[lo:hi], p)
            np.testing.assert_array_equal(alias[lo:hi], a)
        table = (prob, alias)
        del hw
    noise_w = inputs.noise_weights(g.offsets)
    seg = torch.tensor([0, N], dtype=torch.int64, device=DEV)
    noise = gs.gs_alias_build(seg, noise_w)
    o_prob, o_alias = oracle.alias_build(np.array([0, N], dtype=np.int64), noise_w.cpu().numpy())
    np.testing.assert_array_equal(noise.alias.cpu().numpy(), o_alias)
    np.testing.assert_array_equal(noise.prob.cpu().numpy(), o_prob)
    noise_t = (o_prob, o_alias)

    # ---- walks ----------------------------------------------------------------------------
    first = 12_345
    starts = inputs.walk_starts(N, first, num_walks, DEV)
    walks = gs.gs_random_walk(g, row_alias, starts, L, wl.walk_seed, walk_id_base=first)
    h_walks = walks.cpu().numpy()
    h_starts = starts.cpu().numpy()
    for i in np.sort(rng.choice(num_walks, 300, replace=False)):
        want = oracle.random_walk(off, nb, h_starts[i:i + 1], L, wl.walk_seed, alias=table,
                                  walk_id_base=first + int(i))
        np.testing.assert_array_equal(h_walks[i], want[0])

    # ---- pairs ----------------------------------------------------------------------------
    centers, contexts, n_pairs = gs.gs_make_pairs(walks, W)
    lens = (h_walks >= 0).sum(1)
    per = np.where(lens > W, 2 * W * lens - W * (W + 1), lens * (lens - 1))
    assert n_pairs == per.sum() and n_pairs >= B
    base = np.concatenate([[0], np.cumsum(per)])
    hc, ho = centers[:B].cpu().numpy(), contexts[:B].cpu().numpy()
    for i in rng.choice(np.searchsorted(base, B) - 1, 50, replace=False):
        wc, wo = oracle.make_pairs(h_walks[i:i + 1], W)
        np.testing.assert_array_equal(hc[base[i]:base[i + 1]], wc)
        np.testing.assert_array_equal(ho[base[i]:base[i + 1]], wo)

    # ---- negatives ------------------------------------------------------------------------
    pair_base = 11 * B
    negs = gs.gs_sample_negatives(noise, N, B, K, wl.neg_seed, pair_index_base=pair_base)
    hn = negs.cpu().numpy()
    for i in rng.choice(B, 300, replace=False):
        want = oracle.sample_negatives(noise_t, N, 1, K, wl.neg_seed,
                                       pair_index_base=pair_base + int(i))
        np.testing.assert_array_equal(hn[i], want[0])

    # ---- one SGNS iteration at the full batch size -----------------------------------------
    # tables: the workload's initial input table and a context table filled the same way,
    # scaled up so that a wrong or missing term is far outside the tolerance
    w_in, w_out = inputs.init_tables(N, wl.dim, wl.init_seed, DEV, wl.dtype,
                                     context_seed=wl.init_seed + 1)
    w_in.mul_(32.0)
    w_out.mul_(32.0)
    lr = 0.025
    # rows to verify, chosen before the step: busiest destination rows + random ones
    out_ids, out_cnt = np.unique(np.concatenate([ho, hn.ravel()]), return_counts=True)
    pick_out = np.concatenate([out_ids[np.argsort(out_cnt)[-3:]], rng.choice(out_ids, 60, False)])
    cen_ids, cen_cnt = np.unique(hc, return_counts=True)
    pick_cen = np.concatenate([cen_ids[np.argsort(cen_cnt)[-3:]], rng.choice(cen_ids, 60, False)])
    jobs = []
    for r in pick_out:                      # every term of the batch that lands on row r
        as_ctx = ho == r
        as_neg = (hn == r).sum(1)           # a pair may draw the same negative more than once
        ci = np.concatenate([hc[as_ctx], hc[as_neg > 0].repeat(as_neg[as_neg > 0])])
        jobs.append(("out", int(r), ci, int(as_ctx.sum())))
    for c in pick_cen:                      # every pair of the batch centred on c
        sel = np.nonzero(hc == c)[0]
        jobs.append(("in", int(c), sel, 0))
    need_in = np.unique(np.concatenate([j[2] if j[0] == "out" else [j[1]] for j in jobs]))
    need_out = np.unique(np.concatenate(
        [[j[1]] if j[0] == "out" else np.concatenate([ho[j[2]], hn[j[2]].ravel()]) for j in jobs]))
    pre_in = dict(zip(need_in.tolist(), _rows(w_in, need_in)))
    pre_out = dict(zip(need_out.tolist(), _rows(w_out, need_out)))

    # oracle loss over the whole batch (lr = 0 leaves the compacted tables alone)
    want_loss = 0.0
    step = 125_000
    for lo in range(0, B, step):
        hi = min(B, lo + step)
        ids, inv = np.unique(np.concatenate([hc[lo:hi], ho[lo:hi], hn[lo:hi].ravel()]),
                             return_inverse=True)
        inv = inv.astype(np.int32)
        m = hi - lo
        want_loss += oracle.sgns_step(_rows(w_in, ids), _rows(w_out, ids), inv[:m], inv[m:2 * m],
                                      inv[2 * m:].reshape(m, K), 0.0, dtype=odt)

    loss = gs.gs_sgns_step(w_in, w_out, centers[:B], contexts[:B], negs, lr)
    torch.cuda.synchronize()
    got_loss = float(loss.item())
    assert abs(got_loss - want_loss) <= 1e-5 * abs(want_loss)

    zero_row = np.zeros(wl.dim, dtype=np.uint16 if wl.dtype == "bf16" else np.float32)
    tally = [0, 0]                          # bf16: elements not bit-identical, elements checked
    for kind, node, sel, n_ctx in jobs:
        if kind == "out":
            # mini problem: row 0 = the destination row, row 1 = a dummy, rows 2.. = the centres;
            # a context term becomes (centre, context = row 0, negative = dummy) and a negative
            # term (centre, context = dummy, negative = row 0): row 0 receives exactly its terms
            cs = sel
            t_in = np.stack([zero_row, zero_row] + [pre_in[int(c)] for c in cs])
            t_out = np.stack([pre_out[node], zero_row] + [zero_row] * len(cs))
            m_c = np.arange(2, 2 + len(cs), dtype=np.int32)
            m_o = np.where(np.arange(len(cs)) < n_ctx, 0, 1).astype(np.int32)
            m_n = np.where(np.arange(len(cs)) < n_ctx, 1, 0).astype(np.int32)[:, None]
            oracle.sgns_step(t_in, t_out, m_c, m_o, m_n, lr, dtype=odt)
            _check_rows(_rows(w_out, [node])[0], t_out[0], wl.dtype, tally)
        else:
            rows = np.unique(np.concatenate([ho[sel], hn[sel].ravel()]))
            pos = {int(r): k for k, r in enumerate(rows)}
            t_out = np.stack([pre_out[int(r)] for r in rows])
            t_in = np.stack([pre_in[node]] + [zero_row] * (len(rows) - 1)) if len(rows) > 1 \
                else pre_in[node][None, :].copy()
            m_c = np.zeros(len(sel), dtype=np.int32)
            m_o = np.array([pos[int(r)] for r in ho[sel]], dtype=np.int32)
            m_n = np.array([[pos[int(r)] for r in row] for row in hn[sel]], dtype=np.int32)
            oracle.sgns_step(t_in, t_out, m_c, m_o, m_n, lr, dtype=odt)
            _check_rows(_rows(w_in, [node])[0], t_in[0], wl.dtype, tally)

    # elements that rounded the other way (bf16 tables): the same fraction as everywhere
    if tally[1]:
        assert tally[0] <= max(1.0, HALF_FLIP_FRACTION["bf16"] * tally[1]), tally


def test_workload3_full_size(gs, oracle):
    _run_workload(gs, oracle, 3, 12_000)


def test_workload4_full_size(gs, oracle):
    _run_workload(gs, oracle, 4, 400_000)


def test_more_than_2_31_csr_entries(gs, oracle):
    """A regular graph with 40 M nodes and 56 neighbours each: 2.24 G CSR entries, more than
    a 32-bit index holds.  Uniform and node2vec walks on sampled walk ids, LINE samples and
    negatives against the oracle; every position inside the arrays is a 64-bit quantity."""
    n, deg = 40_000_000, 56
    e = n * deg
    assert e > (1 << 31)
    band = n // deg                                             # row r: k * band + (hash(r) mod band), ascending in k
    offsets = torch.arange(n + 1, dtype=torch.int64, device=DEV) * deg
    nbrs = torch.empty(e, dtype=torch.int32, device=DEV)
    chunk = 2_000_000
    ks = (torch.arange(deg, dtype=torch.int64, device=DEV) * band)[None, :]
    for r0 in range(0, n, chunk):
        rows = torch.arange(r0, min(n, r0 + chunk), dtype=torch.int64, device=DEV)
        shift = (rows * 2654435761 % band)[:, None]
        nbrs[r0 * deg:(r0 + rows.numel()) * deg] = (ks + shift).to(torch.int32).reshape(-1)
    g = gs.Csr(offsets, nbrs)
    h_off = offsets.cpu().numpy()
    h_nb = nbrs.cpu().numpy()
    rng = np.random.default_rng(0)
    count, first = 1_000_000, 39_000_000                        # walks that start in the last rows
    starts = torch.arange(first, first + count, dtype=torch.int64, device=DEV).to(torch.int32)
    pick = np.sort(rng.choice(count, 150, replace=False))
    for kind in ("uniform", "node2vec"):
        if kind == "uniform":
            walks = gs.gs_random_walk(g, None, starts, 40, seed=11, walk_id_base=first)
        else:
            walks = gs.gs_node2vec_walk(g, None, starts, 40, 0.5, 2.0, seed=11, walk_id_base=first)
        got = walks[torch.as_tensor(pick, device=DEV)].cpu().numpy()
        for i, row in zip(pick, got):
            s = np.array([first + int(i)], dtype=np.int32)
            if kind == "uniform":
                want = oracle.random_walk(h_off, h_nb, s, 40, seed=11, walk_id_base=first + int(i))
            else:
                want = oracle.node2vec_walk(h_off, h_nb, s, 40, 0.5, 2.0, seed=11,
                                            walk_id_base=first + int(i))
            np.testing.assert_array_equal(row, want[0])
        assert bool((walks >= 0).all())                         # no dead ends in a regular graph
        del walks
    # per-row alias tables over all 2.24 G entries, rows past entry 2^31 against the oracle
    from paper_2407_15452_amd import inputs
    w = torch.empty(e, dtype=torch.float32, device=DEV)
    step = 200_000_000
    for e0 in range(0, e, step):
        idx = torch.arange(e0, min(e, e0 + step), dtype=torch.int64, device=DEV)
        w[e0:e0 + idx.numel()] = ((inputs.hashed_u32(5, idx, 1) >> 8).to(torch.float32) * 2.0 ** -24) ** 3 + 1e-3
        del idx
    table = gs.gs_alias_build(offsets, w, pack=True)
    h_prob, h_alias = table.prob.cpu().numpy(), table.alias.cpu().numpy()
    for r in [0, 1, n // 2, 38_347_923, n - 2, n - 1]:        # 38,347,923 * 56 > 2^31
        seg = np.array([0, deg], dtype=np.int64)
        want_p, want_a = oracle.alias_build(seg, w[r * deg:(r + 1) * deg].cpu().numpy())
        np.testing.assert_array_equal(h_prob[r * deg:(r + 1) * deg], want_p)
        np.testing.assert_array_equal(h_alias[r * deg:(r + 1) * deg], want_a)
    walks = gs.gs_random_walk(g, table, starts, 40, seed=12, walk_id_base=first)
    got = walks[torch.as_tensor(pick, device=DEV)].cpu().numpy()
    for i, row in zip(pick, got):
        want = oracle.random_walk(h_off, h_nb, np.array([first + int(i)], dtype=np.int32), 40, seed=12,
                                  alias=(h_prob, h_alias), walk_id_base=first + int(i))
        np.testing.assert_array_equal(row, want[0])
    del walks, table, w, h_prob, h_alias
    c, o = gs.gs_sample_edges(g, None, 300_000, seed=13, sample_index_base=(1 << 40) + 7)
    want_c, want_o = oracle.sample_edges(h_off, h_nb, 300_000, seed=13,
                                         sample_index_base=(1 << 40) + 7)
    np.testing.assert_array_equal(c.cpu().numpy(), want_c)
    np.testing.assert_array_equal(o.cpu().numpy(), want_o)
    assert int(c.max().item()) > (1 << 31) // deg                # samples from entries past 2^31
