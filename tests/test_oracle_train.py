"""Pins for the oracle's adversarial training step (section 3.2, Algorithm 1, Eq. 5 and 6).

The losses are written as plain formulas; every backward formula is checked against central finite
differences of those losses (float64), and the special cases that have closed forms are checked against
them: an all-zero discriminator (D = 1/2 everywhere), identical draft and target logits (the distillation
gradient vanishes and the loss is the target's entropy), the cross-entropy gradient softmax(d) - softmax(q),
and that one small gradient-descent step lowers the loss it was taken on."""
import copy

import numpy as np
import pytest

from oracle import train as T

H, V, DH, N = 12, 17, 9, 5


def _data(seed, n_fc):
    rng = np.random.default_rng(seed)
    theta = T.disc_params(rng, H, V, DH, n_fc, std=0.4)
    h = rng.normal(size=(N, H))
    q = rng.normal(size=(N, V)) * 2.0
    d = q + rng.normal(size=(N, V))
    return rng, theta, h, q, d


def _fd(f, x, idx, eps=1e-6):
    old = x[idx]
    x[idx] = old + eps
    fp = f()
    x[idx] = old - eps
    fm = f()
    x[idx] = old
    return (fp - fm) / (2 * eps)


def test_losses_written_out_by_hand():
    """Eq. 5 and 6 evaluated with explicit sigmoids, logs and softmaxes on one tiny case."""
    rng, theta, h, q, d = _data(0, 2)
    def D(logits):
        out = []
        for i in range(N):
            u = theta["w_lin"] @ h[i] + logits[i]
            a = np.maximum(theta["w_fc"][0] @ u + theta["b_fc"][0], 0.0)
            s = float(theta["w_fc"][1][0] @ a + theta["b_fc"][1][0])
            out.append(1.0 / (1.0 + np.exp(-s)))
        return np.array(out)
    want_d = -np.mean(np.log(1.0 - D(d))) - np.mean(np.log(D(q)))
    assert T.loss_d(theta, h, q, d) == pytest.approx(want_d, rel=1e-12)
    lam = 0.3
    pq = np.exp(q) / np.exp(q).sum(-1, keepdims=True)
    pd = np.exp(d) / np.exp(d).sum(-1, keepdims=True)
    adv, ce = T.loss_g(theta, h, q, d, lam)
    assert adv == pytest.approx(-lam * np.mean(np.log(D(d))), rel=1e-12)
    assert ce == pytest.approx(np.mean(-(pq * np.log(pd)).sum(-1)), rel=1e-12)


@pytest.mark.parametrize("n_fc", [1, 2, 3])
def test_discriminator_gradients_match_finite_differences(n_fc):
    rng, theta, h, q, d = _data(1 + n_fc, n_fc)
    loss, new, grads = T.disc_step(theta, h, q, d, lr=0.0)
    assert loss == pytest.approx(T.loss_d(theta, h, q, d), rel=1e-13)
    f = lambda: T.loss_d(theta, h, q, d)
    for name in ("w_lin",):
        for _ in range(12):
            idx = tuple(rng.integers(0, s) for s in theta[name].shape)
            assert grads[name][idx] == pytest.approx(_fd(f, theta[name], idx), rel=2e-6, abs=1e-9)
    for k in range(n_fc):
        for name in ("w_fc", "b_fc"):
            for _ in range(8):
                idx = tuple(rng.integers(0, s) for s in theta[name][k].shape)
                assert grads[name][k][idx] == pytest.approx(_fd(f, theta[name][k], idx), rel=2e-6, abs=1e-9)
    # lr = 0 leaves the parameters alone; a positive lr moves them against the gradient
    np.testing.assert_array_equal(new["w_lin"], theta["w_lin"])
    _, moved, _ = T.disc_step(theta, h, q, d, lr=0.5)
    np.testing.assert_allclose(moved["w_fc"][0], theta["w_fc"][0] - 0.5 * grads["w_fc"][0], rtol=1e-13)


@pytest.mark.parametrize("n_fc", [1, 2, 3])
def test_generator_gradient_matches_finite_differences(n_fc):
    rng, theta, h, q, d = _data(10 + n_fc, n_fc)
    lam = 0.7
    adv, ce, g = T.gen_grad(theta, h, q, d, lam)
    assert (adv, ce) == pytest.approx(T.loss_g(theta, h, q, d, lam), rel=1e-13)
    f = lambda: sum(T.loss_g(theta, h, q, d, lam))
    for _ in range(25):
        idx = (int(rng.integers(0, N)), int(rng.integers(0, V)))
        assert g[idx] == pytest.approx(_fd(f, d, idx), rel=2e-6, abs=1e-9)


def test_closed_forms():
    rng, theta, h, q, d = _data(20, 2)
    zero = dict(w_lin=np.zeros_like(theta["w_lin"]), w_fc=[np.zeros_like(w) for w in theta["w_fc"]],
                b_fc=[np.zeros_like(b) for b in theta["b_fc"]])
    # a discriminator that cannot tell anything: D = 1/2, L_D = 2 ln 2, adversarial term = lambda ln 2
    assert T.loss_d(zero, h, q, d) == pytest.approx(2 * np.log(2.0), rel=1e-14)
    adv, ce, g = T.gen_grad(zero, h, q, d, 0.25)
    assert adv == pytest.approx(0.25 * np.log(2.0), rel=1e-14)
    # ... and it passes no gradient back, so dL_G/dd is the cross-entropy's: (softmax(d) - softmax(q)) / N
    sm = lambda x: np.exp(x - x.max(-1, keepdims=True)) / np.exp(x - x.max(-1, keepdims=True)).sum(-1, keepdims=True)
    np.testing.assert_allclose(g, (sm(d) - sm(q)) / N, rtol=1e-12, atol=1e-15)
    # draft == target: the distillation gradient vanishes and the loss is the target's mean entropy
    adv, ce, g = T.gen_grad(zero, h, q, q.copy(), 0.25)
    np.testing.assert_allclose(g, 0.0, atol=1e-15)
    assert ce == pytest.approx(np.mean(-(sm(q) * np.log(sm(q))).sum(-1)), rel=1e-12)
    # lambda = 0 switches the adversarial term off whatever the discriminator is
    adv, _, g0 = T.gen_grad(theta, h, q, d, 0.0)
    assert adv == 0.0
    np.testing.assert_allclose(g0, (sm(d) - sm(q)) / N, rtol=1e-12, atol=1e-15)
    # shifting a logits row by a constant changes no softmax: the distillation gradient sums to zero per row
    np.testing.assert_allclose(g0.sum(-1), 0.0, atol=1e-14)


def test_steps_go_downhill():
    rng, theta, h, q, d = _data(30, 2)
    l0, new, _ = T.disc_step(theta, h, q, d, lr=0.05)
    assert T.loss_d(new, h, q, d) < l0
    adv, ce, g = T.gen_grad(theta, h, q, d, 0.5)
    d2 = d - 0.5 * g
    assert sum(T.loss_g(theta, h, q, d2, 0.5)) < adv + ce


@pytest.mark.parametrize("K", [1, 2, 3])
def test_medusa_head_backward_matches_finite_differences(K):
    """G's own backward pass for a Medusa-style head (K residual blocks, fixed LM head): gradients of
    L_G with respect to the blocks, through the head's forward pass."""
    rng, theta, h, q, _ = _data(40 + K, 2)
    blocks = [rng.normal(size=(H, H)) * 0.3 for _ in range(K)]
    w_lm = rng.normal(size=(V, H)) * 0.5
    lam = 0.4

    def total():
        d, _ = T.medusa_head_forward(blocks, w_lm, h)
        return sum(T.loss_g(theta, h, q, d, lam))
    d, cache = T.medusa_head_forward(blocks, w_lm, h)
    # forward against the definition, row by row
    x = h[2].copy()
    for w in blocks:
        y = w @ x
        x = x + y / (1.0 + np.exp(-y))
    np.testing.assert_allclose(d[2], w_lm @ x, rtol=1e-12)
    _, _, gd = T.gen_grad(theta, h, q, d, lam)
    new, grads = T.medusa_head_step(blocks, w_lm, h, gd, lr=0.1)
    for k in range(K):
        for _ in range(10):
            idx = (int(rng.integers(0, H)), int(rng.integers(0, H)))
            assert grads[k][idx] == pytest.approx(_fd(total, blocks[k], idx), rel=5e-6, abs=1e-9)
        np.testing.assert_allclose(new[k], blocks[k] - 0.1 * grads[k], rtol=1e-13)
    before = total()
    blocks[:] = [b - 0.02 * g for b, g in zip(blocks, grads)]
    assert total() < before
