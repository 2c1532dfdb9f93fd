"""Pins for the oracle's SGNS iteration.

Closed form at the initial state, a hand-computed one-dimensional case, central
finite differences of the loss, dense autograd (the "same result as training
the whole matrix" property of GraphScale §3.2/§4.2), untouched rows, batch
order invariance, and the bf16 storage rule.
"""
import math

import numpy as np
import pytest
import torch


def _batch(rng, n, b, k):
    return (rng.integers(0, n, b).astype(np.int32), rng.integers(0, n, b).astype(np.int32),
            rng.integers(0, n, (b, k)).astype(np.int32))


def _dense_loss(w_in, w_out, c, o, neg):
    """SGNS loss written with torch ops on the full tables (fp64)."""
    u = w_in[torch.as_tensor(c, dtype=torch.long)]
    vp = w_out[torch.as_tensor(o, dtype=torch.long)]
    vn = w_out[torch.as_tensor(neg, dtype=torch.long)]
    pos = torch.nn.functional.softplus(-(u * vp).sum(-1))
    negl = torch.nn.functional.softplus((u[:, None, :] * vn).sum(-1))
    return pos.sum() + negl.sum()


def test_closed_form_at_initial_state(oracle):
    rng = np.random.default_rng(0)
    n, d, b, k, lr = 50, 8, 400, 5, 0.025
    w_in = ((rng.random((n, d)) - 0.5) / d).astype(np.float32)
    w_out = np.zeros((n, d), dtype=np.float32)
    c, o, neg = _batch(rng, n, b, k)
    w_in0 = w_in.copy()
    loss = oracle.sgns_step(w_in, w_out, c, o, neg, lr)
    assert loss == pytest.approx(b * (k + 1) * math.log(2.0), rel=1e-12)
    np.testing.assert_array_equal(w_in, w_in0)          # all context rows were zero
    want = np.zeros((n, d))
    for i in range(b):
        want[o[i]] += 0.5 * lr32(lr) * w_in0[c[i]].astype(np.float64)
        for j in range(k):
            want[neg[i, j]] -= 0.5 * lr32(lr) * w_in0[c[i]].astype(np.float64)
    np.testing.assert_allclose(w_out, want.astype(np.float32), rtol=0, atol=1e-9)


def lr32(lr):
    return float(np.float32(lr))


def test_hand_case_one_dimension(oracle):
    # u = 2, v_ctx = 0.5, v_neg = -1: x0 = 1, x1 = -2
    w_in = np.array([[2.0], [0.0], [0.0]], dtype=np.float32)
    w_out = np.array([[0.0], [0.5], [-1.0]], dtype=np.float32)
    lr = 0.5
    loss = oracle.sgns_step(w_in, w_out, [0], [1], [[2]], lr)
    s = lambda z: 1 / (1 + math.exp(-z))  # noqa: E731
    g0, g1 = s(1.0) - 1, s(-2.0)
    assert loss == pytest.approx(math.log1p(math.exp(-1.0)) + math.log1p(math.exp(-2.0)), rel=1e-14)
    assert w_in[0, 0] == np.float32(2.0 - lr * (g0 * 0.5 + g1 * -1.0))
    assert w_out[1, 0] == np.float32(0.5 - lr * g0 * 2.0)
    assert w_out[2, 0] == np.float32(-1.0 - lr * g1 * 2.0)
    assert w_in[1, 0] == 0 and w_in[2, 0] == 0 and w_out[0, 0] == 0


def test_gradient_matches_finite_differences(oracle):
    rng = np.random.default_rng(1)
    n, d, b, k = 6, 3, 7, 2
    base_in = rng.normal(0, 0.7, (n, d)).astype(np.float32)
    base_out = rng.normal(0, 0.7, (n, d)).astype(np.float32)
    c, o, neg = _batch(rng, n, b, k)

    def loss_at(wi, wo):
        # lr = 0: the call only evaluates the loss
        return oracle.sgns_step(wi.copy(), wo.copy(), c, o, neg, 0.0)

    lr = 1.0
    wi, wo = base_in.copy(), base_out.copy()
    oracle.sgns_step(wi, wo, c, o, neg, lr)
    grad_in = (base_in.astype(np.float64) - wi) / lr     # analytic gradient (fp32-rounded)
    grad_out = (base_out.astype(np.float64) - wo) / lr
    h = 2.0 ** -7                                        # exactly representable perturbation
    for table, grad in ((0, grad_in), (1, grad_out)):
        for r in range(n):
            for e in range(d):
                plus = [base_in.copy(), base_out.copy()]
                minus = [base_in.copy(), base_out.copy()]
                plus[table][r, e] += np.float32(h)
                minus[table][r, e] -= np.float32(h)
                step = float(plus[table][r, e]) - float(minus[table][r, e])
                fd = (loss_at(*plus) - loss_at(*minus)) / step
                assert grad[r, e] == pytest.approx(fd, abs=2e-4), (table, r, e)


def test_matches_dense_autograd_and_leaves_other_rows_alone(oracle):
    rng = np.random.default_rng(2)
    n, d, b, k, lr = 40, 16, 64, 5, 0.025
    w_in = rng.normal(0, 0.5, (n, d)).astype(np.float32)
    w_out = rng.normal(0, 0.5, (n, d)).astype(np.float32)
    c, o, neg = _batch(rng, 25, b, k)                    # rows 25..39 never named
    ti = torch.tensor(w_in, dtype=torch.float64, requires_grad=True)
    to = torch.tensor(w_out, dtype=torch.float64, requires_grad=True)
    dense = _dense_loss(ti, to, c, o, neg)
    dense.backward()
    before_in, before_out = w_in.copy(), w_out.copy()
    loss = oracle.sgns_step(w_in, w_out, c, o, neg, lr)
    assert loss == pytest.approx(dense.item(), rel=1e-12)
    want_in = (before_in.astype(np.float64) - lr32(lr) * ti.grad.numpy()).astype(np.float32)
    want_out = (before_out.astype(np.float64) - lr32(lr) * to.grad.numpy()).astype(np.float32)
    # identical up to the order of fp64 additions before the single fp32 rounding
    np.testing.assert_allclose(w_in, want_in, rtol=0, atol=1e-7)
    np.testing.assert_allclose(w_out, want_out, rtol=0, atol=1e-7)
    assert (ti.grad[25:] == 0).all() and (to.grad[25:] == 0).all()
    np.testing.assert_array_equal(w_in[25:], before_in[25:])
    np.testing.assert_array_equal(w_out[25:], before_out[25:])
    touched_in = np.zeros(n, bool)
    touched_in[c] = True
    np.testing.assert_array_equal(w_in[~touched_in], before_in[~touched_in])


def test_reads_see_pre_step_values(oracle):
    # the same row is centre of one pair and context of another, and is hit twice:
    # a sequential (pair-by-pair) update would give a different answer
    w_in = np.array([[1.0, 0.5], [0.25, -1.0]], dtype=np.float32)
    w_out = np.array([[0.5, 0.5], [-0.5, 1.0]], dtype=np.float32)
    c = np.array([0, 1, 0], dtype=np.int32)
    o = np.array([1, 0, 1], dtype=np.int32)
    neg = np.array([[0], [1], [0]], dtype=np.int32)
    ti = torch.tensor(w_in, dtype=torch.float64, requires_grad=True)
    to = torch.tensor(w_out, dtype=torch.float64, requires_grad=True)
    _dense_loss(ti, to, c, o, neg).backward()
    a, b = w_in.copy(), w_out.copy()
    oracle.sgns_step(a, b, c, o, neg, 0.5)
    np.testing.assert_allclose(a, w_in - 0.5 * ti.grad.numpy(), atol=1e-7)
    np.testing.assert_allclose(b, w_out - 0.5 * to.grad.numpy(), atol=1e-7)


def test_batch_order_does_not_matter(oracle):
    rng = np.random.default_rng(3)
    n, d, b, k = 30, 8, 200, 3
    w_in = rng.normal(0, 0.5, (n, d)).astype(np.float32)
    w_out = rng.normal(0, 0.5, (n, d)).astype(np.float32)
    c, o, neg = _batch(rng, n, b, k)
    a_in, a_out = w_in.copy(), w_out.copy()
    la = oracle.sgns_step(a_in, a_out, c, o, neg, 0.025)
    perm = rng.permutation(b)
    b_in, b_out = w_in.copy(), w_out.copy()
    lb = oracle.sgns_step(b_in, b_out, c[perm], o[perm], neg[perm], 0.025)
    assert la == pytest.approx(lb, rel=1e-13)
    np.testing.assert_allclose(a_in, b_in, rtol=0, atol=1e-7)
    np.testing.assert_allclose(a_out, b_out, rtol=0, atol=1e-7)


def test_empty_batch_and_zero_negatives(oracle):
    w_in = np.ones((3, 4), dtype=np.float32)
    w_out = np.ones((3, 4), dtype=np.float32)
    e = np.zeros(0, dtype=np.int32)
    assert oracle.sgns_step(w_in, w_out, e, e, np.zeros((0, 5), dtype=np.int32), 0.1) == 0.0
    assert (w_in == 1).all() and (w_out == 1).all()
    loss = oracle.sgns_step(w_in, w_out, [0], [1], np.zeros((1, 0), dtype=np.int32), 0.1)
    assert loss == pytest.approx(math.log1p(math.exp(-4.0)), rel=1e-14)


def test_bf16_tables_round_to_nearest_even_once(oracle):
    rng = np.random.default_rng(4)
    n, d, b, k, lr = 20, 8, 100, 4, 0.05
    f_in = torch.tensor(rng.normal(0, 0.5, (n, d)), dtype=torch.float32).to(torch.bfloat16)
    f_out = torch.tensor(rng.normal(0, 0.5, (n, d)), dtype=torch.float32).to(torch.bfloat16)
    c, o, neg = _batch(rng, n, b, k)
    bits_in = f_in.view(torch.int16).numpy().view(np.uint16).copy()
    bits_out = f_out.view(torch.int16).numpy().view(np.uint16).copy()
    # the same step on exactly widened fp32 copies
    w_in = f_in.to(torch.float32).numpy().copy()
    w_out = f_out.to(torch.float32).numpy().copy()
    l32 = oracle.sgns_step(w_in, w_out, c, o, neg, lr)
    l16 = oracle.sgns_step(bits_in, bits_out, c, o, neg, lr, dtype=oracle.BF16)
    assert l16 == l32                                    # reads widen exactly
    want_in = torch.tensor(w_in).to(torch.bfloat16)      # torch rounds to nearest even
    want_out = torch.tensor(w_out).to(torch.bfloat16)
    got_in = torch.from_numpy(bits_in.view(np.int16)).view(torch.bfloat16)
    got_out = torch.from_numpy(bits_out.view(np.int16)).view(torch.bfloat16)
    assert torch.equal(got_in, want_in) and torch.equal(got_out, want_out)


def test_f16_conversions_match_numpy(oracle):
    """binary16 storage: every bit pattern widens as numpy's float16 does; fp32 -> binary16
    rounds to nearest even like numpy, subnormals, ties, overflow and signed zero included."""
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.f16_to_float(bits)
    want = bits.view(np.float16).astype(np.float32)
    finite = np.isfinite(want)
    np.testing.assert_array_equal(got[finite], want[finite])
    np.testing.assert_array_equal(np.isnan(got), np.isnan(want))
    np.testing.assert_array_equal(got[np.isinf(want)], want[np.isinf(want)])
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.normal(0, 1, 100_000), rng.normal(0, 1e-6, 50_000),
                        rng.normal(0, 3e4, 50_000),
                        [0.0, -0.0, 65504, 65519.99, 65520, 1e9, -1e9, 6e-8, 2.98e-8, 2.9802322e-8,
                         5.96e-8, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, np.inf, -np.inf]]).astype(np.float32)
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    np.testing.assert_array_equal(oracle.float_to_f16(x), want)


def test_f16_tables_round_to_nearest_even_once(oracle):
    rng = np.random.default_rng(14)
    n, d, b, k, lr = 20, 8, 100, 4, 0.05
    f_in = rng.normal(0, 0.5, (n, d)).astype(np.float16)
    f_out = rng.normal(0, 0.5, (n, d)).astype(np.float16)
    c, o, neg = _batch(rng, n, b, k)
    bits_in, bits_out = f_in.view(np.uint16).copy(), f_out.view(np.uint16).copy()
    w_in, w_out = f_in.astype(np.float32), f_out.astype(np.float32)   # exactly widened copies
    l32 = oracle.sgns_step(w_in, w_out, c, o, neg, lr)
    l16 = oracle.sgns_step(bits_in, bits_out, c, o, neg, lr, dtype=oracle.F16)
    assert l16 == l32
    np.testing.assert_array_equal(bits_in, w_in.astype(np.float16).view(np.uint16))
    np.testing.assert_array_equal(bits_out, w_out.astype(np.float16).view(np.uint16))


# ----------------------------------------------------------------------------- SGD with momentum
def test_momentum_step_matches_torch_sgd(oracle):
    """mult / put / mult_add (GraphScale §3.2) is torch.optim.SGD(momentum=mu) on the dense
    tables: buf = mu * buf + grad, p -= lr * buf.  Three iterations on different batches."""
    rng = np.random.default_rng(7)
    n, d, b, k, lr, mu = 30, 8, 40, 3, 0.05, 0.9
    w_in = rng.normal(0, 0.5, (n, d)).astype(np.float32)
    w_out = rng.normal(0, 0.5, (n, d)).astype(np.float32)
    m_in = np.zeros((n, d), dtype=np.float32)
    m_out = np.zeros((n, d), dtype=np.float32)
    ti = torch.tensor(w_in, dtype=torch.float64, requires_grad=True)
    to = torch.tensor(w_out, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([ti, to], lr=float(np.float32(lr)), momentum=float(np.float32(mu)))
    for it in range(3):
        c, o, neg = _batch(rng, 20, b, k)                # rows 20..29 are never named
        opt.zero_grad()
        dense = _dense_loss(ti, to, c, o, neg)
        dense.backward()
        opt.step()
        loss = oracle.sgns_momentum_step(w_in, w_out, m_in, m_out, c, o, neg, lr, mu)
        assert loss == pytest.approx(dense.item(), rel=1e-6)
        np.testing.assert_allclose(w_in, ti.detach().numpy(), atol=2e-6)
        np.testing.assert_allclose(w_out, to.detach().numpy(), atol=2e-6)
        np.testing.assert_allclose(m_in, opt.state[ti]["momentum_buffer"].numpy(), atol=2e-6)
        np.testing.assert_allclose(m_out, opt.state[to]["momentum_buffer"].numpy(), atol=2e-6)
    assert (m_in[20:] == 0).all() and np.abs(m_in[:20]).max() > 0


def test_momentum_step_without_momentum_is_plain_sgd(oracle):
    rng = np.random.default_rng(8)
    n, d, b, k, lr = 25, 4, 60, 2, 0.1
    w_in = rng.normal(0, 0.5, (n, d)).astype(np.float32)
    w_out = rng.normal(0, 0.5, (n, d)).astype(np.float32)
    c, o, neg = _batch(rng, n, b, k)
    a_in, a_out = w_in.copy(), w_out.copy()
    la = oracle.sgns_step(a_in, a_out, c, o, neg, lr)
    m_in = rng.normal(0, 1, (n, d)).astype(np.float32)   # wiped by mu = 0
    m_out = rng.normal(0, 1, (n, d)).astype(np.float32)
    lb = oracle.sgns_momentum_step(w_in, w_out, m_in, m_out, c, o, neg, lr, 0.0)
    assert la == lb
    # w - lr * round32(G) against round32(w - lr * G): one extra fp32 rounding of the gradient
    np.testing.assert_allclose(w_in, a_in, atol=1e-6)
    np.testing.assert_allclose(w_out, a_out, atol=1e-6)


def test_momentum_step_moves_every_row_with_momentum(oracle):
    # a row the batch does not name still moves by -lr * mu * momentum (the dense mult_add)
    w_in = np.ones((4, 2), dtype=np.float32)
    w_out = np.ones((4, 2), dtype=np.float32)
    m_in = np.full((4, 2), 0.5, dtype=np.float32)
    m_out = np.full((4, 2), -0.25, dtype=np.float32)
    oracle.sgns_momentum_step(w_in, w_out, m_in, m_out, [0], [1], np.array([[1]], dtype=np.int32),
                              0.5, 0.5)
    assert m_in[3, 0] == 0.25 and m_out[3, 0] == -0.125
    assert w_in[3, 0] == 1.0 - 0.5 * 0.25 and w_out[3, 0] == 1.0 + 0.5 * 0.125


def test_adam_step_matches_torch_adam(oracle):
    """mult / put / apply over the storage is torch.optim.Adam on the dense tables (gradient
    zero outside the batch).  Four iterations on different batches, state compared too."""
    rng = np.random.default_rng(17)
    n, d, b, k = 30, 8, 40, 3
    lr, b1, b2, eps = 0.01, 0.9, 0.999, 1e-8
    w_in = rng.normal(0, 0.5, (n, d)).astype(np.float32)
    w_out = rng.normal(0, 0.5, (n, d)).astype(np.float32)
    m_in, m_out, v_in, v_out = (np.zeros((n, d), dtype=np.float32) for _ in range(4))
    ti = torch.tensor(w_in, dtype=torch.float64, requires_grad=True)
    to = torch.tensor(w_out, dtype=torch.float64, requires_grad=True)
    f = lambda x: float(np.float32(x))
    opt = torch.optim.Adam([ti, to], lr=f(lr), betas=(f(b1), f(b2)), eps=f(eps))
    for it in range(1, 5):
        c, o, neg = _batch(rng, 20, b, k)                # rows 20..29 are never named
        opt.zero_grad()
        dense = _dense_loss(ti, to, c, o, neg)
        dense.backward()
        opt.step()
        loss = oracle.sgns_adam_step(w_in, w_out, m_in, m_out, v_in, v_out, c, o, neg, lr, b1, b2,
                                     eps, it)
        assert loss == pytest.approx(dense.item(), rel=1e-6)
        np.testing.assert_allclose(w_in, ti.detach().numpy(), atol=2e-6)
        np.testing.assert_allclose(w_out, to.detach().numpy(), atol=2e-6)
        np.testing.assert_allclose(m_in, opt.state[ti]["exp_avg"].numpy(), rtol=1e-5, atol=1e-7)
        np.testing.assert_allclose(v_out, opt.state[to]["exp_avg_sq"].numpy(), rtol=1e-5, atol=1e-9)
    assert (m_in[20:] == 0).all() and (v_in[20:] == 0).all() and np.abs(m_in[:20]).max() > 0
    np.testing.assert_array_equal(w_in[20:], ti.detach().numpy()[20:].astype(np.float32))


def test_adam_first_step_has_magnitude_lr(oracle):
    # t = 1: m / (1 - b1) = g, sqrt(v / (1 - b2)) = |g|, so every touched element moves by lr * sign(g)
    rng = np.random.default_rng(18)
    n, d, lr = 12, 4, 0.05
    w_in = rng.normal(0, 0.5, (n, d)).astype(np.float32)
    w_out = rng.normal(0, 0.5, (n, d)).astype(np.float32)
    c, o, neg = _batch(rng, n, 30, 2)
    a_in, a_out = w_in.copy(), w_out.copy()
    oracle.sgns_step(a_in, a_out, c, o, neg, 1.0)        # a - w = -gradient
    z = [np.zeros((n, d), dtype=np.float32) for _ in range(4)]
    b_in, b_out = w_in.copy(), w_out.copy()
    oracle.sgns_adam_step(b_in, b_out, *z, c, o, neg, lr, 0.9, 0.999, 1e-12, 1)
    for before, sgd, adam in ((w_in, a_in, b_in), (w_out, a_out, b_out)):
        g = before.astype(np.float64) - sgd
        big = np.abs(g) > 1e-3
        np.testing.assert_allclose((adam - before)[big], -lr * np.sign(g[big]), rtol=1e-4)
        assert ((adam - before)[g == 0] == 0).all()


def test_adam_decays_state_of_rows_outside_the_batch(oracle):
    # the dense passes: an unnamed row keeps moving along its decayed first moment
    w_in = np.ones((4, 2), dtype=np.float32)
    w_out = np.ones((4, 2), dtype=np.float32)
    m_in = np.full((4, 2), 0.5, dtype=np.float32); m_out = m_in.copy()
    v_in = np.full((4, 2), 0.25, dtype=np.float32); v_out = v_in.copy()
    oracle.sgns_adam_step(w_in, w_out, m_in, m_out, v_in, v_out, [0], [1],
                          np.array([[1]], dtype=np.int32), 0.1, 0.5, 0.5, 0.0, 1)
    assert m_in[3, 0] == 0.25 and v_in[3, 0] == 0.125
    # step = lr / (1 - 0.5) = 0.2; denominator sqrt(0.125) / sqrt(0.5) = 0.5
    assert w_in[3, 0] == pytest.approx(1.0 - 0.2 * 0.25 / 0.5, abs=1e-7)
