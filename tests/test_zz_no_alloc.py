"""gs_sgns_step_static: the step on the library's static scratch array (no workspace argument,
nothing allocated by the call) against gs_sgns_step on a caller workspace.  Both add the terms
of a row exactly, so the tables and the loss must agree bit for bit; two calls in a row, the
second with a smaller batch (the array keeps the first call's contents)."""
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
    binding.lib()
    return binding


def _batch(rng, n, b, k):
    c = np.repeat((n * rng.random(b // 4 + 1) ** 2).astype(np.int32), 4)[:b]
    o = rng.integers(0, n, b).astype(np.int32)
    neg = (n * rng.random((b, k)) ** 5).astype(np.int32)        # hub rows: long rows of terms
    return [torch.as_tensor(x).to(DEV) for x in (c, o, neg)]


@pytest.mark.parametrize("fmt", ["f32", "bf16"])
def test_static_step_matches_workspace_step(gs, fmt):
    from paper_2407_15452_amd import inputs
    n, dim = 50_000, 128
    f_in, f_out = inputs.random_tables(n, dim, seed=3, scale=0.2)
    tdt = torch.float32 if fmt == "f32" else torch.bfloat16
    bits = torch.int32 if fmt == "f32" else torch.int16
    rng = np.random.default_rng(17)
    a_in, a_out = f_in.to(tdt).to(DEV), f_out.to(tdt).to(DEV)      # static scratch
    b_in, b_out = a_in.clone(), a_out.clone()                      # caller workspace
    loss_a = torch.zeros(1, dtype=torch.float64, device=DEV)
    loss_b = torch.zeros(1, dtype=torch.float64, device=DEV)
    for b, k in ((4096, 15), (700, 5), (1, 0)):                    # largest allowed, then smaller ones
        c, o, neg = _batch(rng, n, b, k)
        gs.gs_sgns_step_static(a_in, a_out, c, o, neg, 0.025, loss_out=loss_a)
        gs.gs_sgns_step(b_in, b_out, c, o, neg, 0.025, loss_out=loss_b)
        torch.cuda.synchronize()
        assert torch.equal(loss_a.view(torch.int64), loss_b.view(torch.int64))
        assert torch.equal(a_in.view(bits), b_in.view(bits))
        assert torch.equal(a_out.view(bits), b_out.view(bits))
    assert not torch.equal(a_out.view(bits), f_out.to(tdt).to(DEV).view(bits))   # it did train


def test_static_step_rejects_what_does_not_fit(gs):
    w = [torch.zeros((100, 64), dtype=torch.float32, device=DEV) for _ in range(2)]
    big = torch.zeros(4097, dtype=torch.int32, device=DEV)
    with pytest.raises(gs.GsError) as err:
        gs.gs_sgns_step_static(w[0], w[1], big, big, torch.zeros((4097, 1), dtype=torch.int32, device=DEV), 0.1)
    assert err.value.status == gs.GS_EWORKSPACE
    ids = torch.zeros(4096, dtype=torch.int32, device=DEV)
    with pytest.raises(gs.GsError) as err:                              # 4096 * 17 terms
        gs.gs_sgns_step_static(w[0], w[1], ids, ids, torch.zeros((4096, 16), dtype=torch.int32, device=DEV), 0.1)
    assert err.value.status == gs.GS_EWORKSPACE
    wide = [torch.zeros((100, 512), dtype=torch.float32, device=DEV) for _ in range(2)]
    with pytest.raises(gs.GsError) as err:
        gs.gs_sgns_step_static(wide[0], wide[1], ids[:8], ids[:8], torch.zeros((8, 1), dtype=torch.int32, device=DEV), 0.1)
    assert err.value.status == gs.GS_EWORKSPACE


def test_static_step_replays_from_a_captured_graph(gs):
    """The use the entry point is for: captured once into a HIP graph (nothing is allocated,
    the scratch array is cleared by a kernel), replayed on fresh batches with eager work and
    synchronisation between the replays; every replay against the eager gs_sgns_step, bit for
    bit.  The address of the scratch array is looked up by the warm-up call outside the capture."""
    from paper_2407_15452_amd import inputs
    n, dim, b, k = 30_000, 64, 2_048, 5
    f_in, f_out = inputs.random_tables(n, dim, seed=9, scale=0.2)
    a_in, a_out = f_in.to(DEV), f_out.to(DEV)
    b_in, b_out = a_in.clone(), a_out.clone()
    c_buf = torch.zeros(b, dtype=torch.int32, device=DEV)
    o_buf = torch.zeros(b, dtype=torch.int32, device=DEV)
    n_buf = torch.zeros((b, k), dtype=torch.int32, device=DEV)
    loss_a = torch.zeros(1, dtype=torch.float64, device=DEV)
    loss_b = torch.zeros(1, dtype=torch.float64, device=DEV)

    def body():
        gs.gs_sgns_step_static(a_in, a_out, c_buf, o_buf, n_buf, 0.025, loss_out=loss_a)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        body()                                   # warm-up outside capture (ids 0)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        body()
    a_in.copy_(b_in); a_out.copy_(b_out)         # capture does not run the kernels; start equal
    rng = np.random.default_rng(23)
    for it in range(3):
        c, o, neg = _batch(rng, n, b, k)
        c_buf.copy_(c); o_buf.copy_(o); n_buf.copy_(neg)
        graph.replay()
        gs.gs_sgns_step(b_in, b_out, c, o, neg, 0.025, loss_out=loss_b)
        torch.cuda.synchronize()
        assert torch.equal(loss_a.view(torch.int64), loss_b.view(torch.int64))
        assert torch.equal(a_in.view(torch.int32), b_in.view(torch.int32))
        assert torch.equal(a_out.view(torch.int32), b_out.view(torch.int32))
        _ = (a_in * 2).sum().item()              # eager work of the program's own between the replays
