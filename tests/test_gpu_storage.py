"""GPU parity for the storage operations on a batch of ids (gs_unique_ids,
gs_get_rows, gs_put_rows) against the oracle: ids and positions bit-exact, fetched
rows bit-exact, written rows bit-exact (both sides round the exact sum once)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def gs():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2407_15452_amd import binding
    binding.lib()          # raises if libgs.so was not built
    return binding


def _t(a):
    return torch.as_tensor(np.ascontiguousarray(a)).to(DEV)


def _bits(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("n,num_nodes,bad", [(0, 10, False), (1, 10, False), (4097, 300, False),
                                             (100_003, 1_000_000, True), (250_000, 5_000, False),
                                             (70_001, (1 << 31) - 1, True)])
def test_unique_ids(gs, oracle, n, num_nodes, bad):
    rng = np.random.default_rng(n)
    ids = rng.integers(0, min(num_nodes, 1 << 20), n).astype(np.int32)
    if num_nodes > (1 << 20) and n:
        ids[::3] = rng.integers(0, num_nodes, ids[::3].size)       # use the high bits too
    if bad and n:
        ids[rng.random(n) < 0.01] = -5
        if num_nodes < (1 << 31) - 1:
            ids[rng.random(n) < 0.01] = num_nodes
    want_u, want_inv = oracle.unique_ids(ids, num_nodes)
    u, count, inv = gs.gs_unique_ids(_t(ids).reshape(-1), num_nodes)
    k = int(count.item())
    assert k == want_u.size
    np.testing.assert_array_equal(u[:k].cpu().numpy(), want_u)
    np.testing.assert_array_equal(inv.cpu().numpy(), want_inv)
    u2, count2, inv2 = gs.gs_unique_ids(_t(ids).reshape(-1), num_nodes, want_inverse=False)
    assert inv2 is None and int(count2.item()) == k
    np.testing.assert_array_equal(u2[:k].cpu().numpy(), want_u)


@pytest.mark.parametrize("dtype,dim", [("f32", 128), ("f32", 4), ("f32", 100), ("bf16", 256),
                                       ("bf16", 8), ("bf16", 72), ("f32", 1024), ("f16", 128),
                                       ("f16", 8)])
def test_get_and_put_rows(gs, oracle, dtype, dim):
    from paper_2407_15452_amd import inputs
    n_nodes, n = 20_011, 7_003
    rng = np.random.default_rng(dim)
    table = inputs.random_tables(n_nodes, dim, 5, 0.5)[0]
    ids = rng.permutation(n_nodes)[:n].astype(np.int32)
    ids[5], ids[77] = -1, n_nodes                                   # not rows: zero / skipped
    rows = rng.normal(size=(n, dim)).astype(np.float32)
    if dtype in ("bf16", "f16"):
        d_table = table.to(torch.bfloat16 if dtype == "bf16" else torch.float16).to(DEV)
        h_table = _bits(d_table).copy()
        code = oracle.BF16 if dtype == "bf16" else oracle.F16
    else:
        d_table = table.to(DEV)
        h_table = table.numpy().copy()
        code = oracle.F32
    got = gs.gs_get_rows(d_table, _t(ids))
    np.testing.assert_array_equal(got.cpu().numpy(), oracle.get_rows(h_table, ids, dtype=code))
    gs.gs_put_rows(d_table, _t(ids), _t(rows), -0.37)
    oracle.put_rows(h_table, ids, rows, -0.37, dtype=code)
    after = _bits(d_table) if dtype != "f32" else d_table.cpu().numpy()
    np.testing.assert_array_equal(after, h_table)


def test_count_on_device_limits_the_rows(gs, oracle):
    from paper_2407_15452_amd import inputs
    n_nodes, dim = 5_000, 64
    table = inputs.random_tables(n_nodes, dim, 6, 0.5)[0]
    rng = np.random.default_rng(1)
    batch = rng.integers(0, n_nodes, 30_000).astype(np.int32)
    u, count, inv = gs.gs_unique_ids(_t(batch), n_nodes)
    k = int(count.item())
    assert k < batch.size
    d_table = table.to(DEV)
    out = torch.full((batch.size, dim), 7.0, dtype=torch.float32, device=DEV)
    gs.gs_get_rows(d_table, u, count=count, out=out)
    want_u, _ = oracle.unique_ids(batch, n_nodes)
    np.testing.assert_array_equal(out[:k].cpu().numpy(), table.numpy()[want_u])
    assert (out[k:] == 7.0).all()                                  # rows past the count are not written
    gs.gs_put_rows(d_table, u, out, 2.0, count=count)
    h = table.numpy().copy()
    oracle.put_rows(h, want_u, table.numpy()[want_u], 2.0)
    np.testing.assert_array_equal(d_table.cpu().numpy(), h)


def test_block_step_equals_full_table_step(gs, oracle):
    """unique -> get -> step on the n x d block -> put of the deltas gives the rows of the
    step on the full tables (the sparse update of the paper) within the SGNS tolerance."""
    from paper_2407_15452_amd import inputs
    n_nodes, dim, B, K = 30_000, 64, 8_192, 5
    w_in, w_out = inputs.random_tables(n_nodes, dim, 8, 0.3)
    rng = np.random.default_rng(2)
    c = rng.integers(0, n_nodes, B).astype(np.int32)
    o = rng.integers(0, n_nodes, B).astype(np.int32)
    neg = rng.integers(0, n_nodes, (B, K)).astype(np.int32)
    full_in, full_out = w_in.to(DEV), w_out.to(DEV)
    gs.gs_sgns_step(full_in, full_out, _t(c), _t(o), _t(neg), 0.05)
    ids = _t(np.concatenate([c, o, neg.ravel()]))
    u, count, inv = gs.gs_unique_ids(ids, n_nodes)
    k = int(count.item())
    d_in, d_out = w_in.to(DEV), w_out.to(DEV)
    blk_in, blk_out = gs.gs_get_rows(d_in, u[:k]), gs.gs_get_rows(d_out, u[:k])
    new_in, new_out = blk_in.clone(), blk_out.clone()
    gs.gs_sgns_step(new_in, new_out, inv[:B].contiguous(), inv[B:2 * B].contiguous(),
                    inv[2 * B:].reshape(B, K).contiguous(), 0.05)
    gs.gs_put_rows(d_in, u[:k], new_in - blk_in, 1.0)
    gs.gs_put_rows(d_out, u[:k], new_out - blk_out, 1.0)
    assert (d_in - full_in).abs().max().item() <= 1e-5
    assert (d_out - full_out).abs().max().item() <= 1e-5


def test_storage_argument_errors(gs):
    t = torch.zeros((10, 6), dtype=torch.float32, device=DEV)      # dim not a multiple of 4
    ids = torch.zeros(3, dtype=torch.int32, device=DEV)
    with pytest.raises(gs.GsError):
        gs.gs_get_rows(t, ids)
    with pytest.raises(gs.GsError):
        gs.gs_put_rows(t, ids, torch.zeros((3, 6), device=DEV), 1.0)
    with pytest.raises(gs.GsError):
        gs.gs_unique_ids(ids, 0)
    small = torch.empty(256, dtype=torch.uint8, device=DEV)
    with pytest.raises(gs.GsError):
        gs.gs_unique_ids(torch.zeros(100_000, dtype=torch.int32, device=DEV), 10, ws=small)


@pytest.mark.parametrize("dtype,dim", [("f32", 128), ("f32", 4), ("bf16", 256), ("bf16", 8),
                                       ("f16", 64)])
def test_dense_mult_and_mult_add(gs, oracle, dtype, dim):
    from paper_2407_15452_amd import inputs
    n = 30_011
    a, b = inputs.random_tables(n, dim, 9, 1.5)
    if dtype in ("bf16", "f16"):
        tdt = torch.bfloat16 if dtype == "bf16" else torch.float16
        d_a, d_b = a.to(tdt).to(DEV), b.to(tdt).to(DEV)
        h_a, h_b = _bits(d_a).copy(), _bits(d_b).copy()
        code = oracle.BF16 if dtype == "bf16" else oracle.F16
    else:
        d_a, d_b = a.to(DEV), b.to(DEV)
        h_a, h_b = a.numpy().copy(), b.numpy().copy()
        code = oracle.F32
    gs.gs_table_mult(d_a, 0.9)
    oracle.table_mult(h_a, 0.9, dtype=code)
    gs.gs_table_mult_add(d_b, d_a, -0.025)
    oracle.table_mult_add(h_b, h_a, -0.025, dtype=code)
    view = _bits if dtype != "f32" else (lambda t: t.cpu().numpy())
    np.testing.assert_array_equal(view(d_a), h_a)
    np.testing.assert_array_equal(view(d_b), h_b)
    with pytest.raises(gs.GsError):
        gs.gs_table_mult_add(d_a, d_a, 1.0)


def test_momentum_update_from_the_storage_operations(gs, oracle):
    """mult, put of the gradient rows, mult_add: the paper's model update composed from the
    exported operations, against gs_sgns_momentum_step."""
    from paper_2407_15452_amd import inputs
    n, d, B, K, lr, mu = 20_000, 64, 8_192, 5, 0.05, 0.9
    w_in, w_out = inputs.random_tables(n, d, 8, 0.3)
    m_in, m_out = inputs.random_tables(n, d, 9, 0.05)
    rng = np.random.default_rng(2)
    c = _t(rng.integers(0, n, B).astype(np.int32))
    o = _t(rng.integers(0, n, B).astype(np.int32))
    neg = _t(rng.integers(0, n, (B, K)).astype(np.int32))
    want = [t.to(DEV) for t in (w_in, w_out, m_in, m_out)]
    gs.gs_sgns_momentum_step(*want, c, o, neg, lr, mu)
    got = [t.to(DEV) for t in (w_in, w_out, m_in, m_out)]
    # gradient rows of the batch: a plain step with lr = 1 on copies, old - new
    s_in, s_out = got[0].clone(), got[1].clone()
    gs.gs_sgns_step(s_in, s_out, c, o, neg, 1.0)
    for model, moment, stepped, ids in ((got[0], got[2], s_in, c),
                                        (got[1], got[3], s_out, torch.cat([o, neg.reshape(-1)]))):
        u, count, _ = gs.gs_unique_ids(ids, n, want_inverse=False)
        grads = gs.gs_get_rows(model, u, count=count) - gs.gs_get_rows(stepped, u, count=count)
        gs.gs_table_mult(moment, mu)
        gs.gs_put_rows(moment, u, grads, 1.0, count=count)
        gs.gs_table_mult_add(model, moment, -lr)
    for g_t, w_t in zip(got, want):
        assert (g_t - w_t).abs().max().item() <= 1e-5
