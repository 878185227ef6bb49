"""GPU parity of the adversarial training step (section 3.2, Algorithm 1, Eq. 5 and 6) against the oracle:
losses, the gradient at the draft logits, and every parameter after one gradient-descent update, for
discriminators of one, two and three fully connected layers and Medusa-style heads of K = 1..3 blocks.
fp32 on the device against fp64 on the CPU: 1e-4 of the largest reference magnitude per tensor; updated
parameters are compared through the update itself (new - old), so that a wrong gradient cannot hide
behind the size of the weights."""
import numpy as np
import pytest

from oracle import train as T

pytestmark = pytest.mark.gpu

TOL = 1e-4


def _close(got, ref, what):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    err = np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30)
    assert err < TOL, f"{what}: relative error {err:.2e}"


def _setup(seed, H, V, DH, n_fc, N):
    import torch
    rng = np.random.default_rng(seed)
    theta = T.disc_params(rng, H, V, DH, n_fc, std=0.05)
    h = rng.normal(size=(N, H))
    q = rng.normal(size=(N, V)) * 2.0
    d = q + rng.normal(size=(N, V))
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return rng, theta, h, q, d, dev


# sizes: several 64-wide GEMM tiles with ragged edges in every dimension, K not a multiple of 16
@pytest.mark.parametrize("n_fc,H,V,DH,N", [(1, 200, 1000, 0, 37), (2, 200, 1000, 150, 37), (3, 136, 777, 90, 70)])
def test_discriminator_step_matches_oracle(n_fc, H, V, DH, N):
    import torch
    import paper_2408_08146_amd as K
    rng, theta, h, q, d, dev = _setup(3 + n_fc, H, V, max(DH, 1), n_fc, N)
    lr = 0.3
    loss_ref, new, grads = T.disc_step(theta, h, q, d, lr)
    w_lin = dev(theta["w_lin"])
    w_fc = [dev(w) for w in theta["w_fc"]]
    b_fc = [dev(b) for b in theta["b_fc"]]
    D = K.Discriminator(w_lin, w_fc, b_fc, fc_hidden=DH)
    loss = torch.zeros(1, device="cuda")
    D.step(dev(h), dev(q), dev(d), lr, loss)
    torch.cuda.synchronize()
    assert abs(loss.item() - loss_ref) < TOL * abs(loss_ref)
    _close((w_lin.cpu().numpy() - theta["w_lin"].astype(np.float32)), -lr * grads["w_lin"], "w_lin update")
    for k in range(n_fc):
        _close(w_fc[k].cpu().numpy() - theta["w_fc"][k].astype(np.float32), -lr * grads["w_fc"][k], f"w_fc[{k}] update")
        _close(b_fc[k].cpu().numpy() - theta["b_fc"][k].astype(np.float32), -lr * grads["b_fc"][k], f"b_fc[{k}] update")
    # lr = 0: loss only, nothing moves
    before = w_fc[0].clone()
    D.step(dev(h), dev(q), dev(d), 0.0, loss)
    torch.cuda.synchronize()
    assert torch.equal(before, w_fc[0])
    assert abs(loss.item() - T.loss_d(new, h, q, d)) < 5 * TOL * abs(loss_ref)


@pytest.mark.parametrize("n_fc,H,V,DH,N", [(1, 200, 1000, 0, 37), (2, 200, 1000, 150, 37), (3, 136, 777, 90, 70)])
def test_generator_loss_and_gradient_match_oracle(n_fc, H, V, DH, N):
    import torch
    import paper_2408_08146_amd as K
    rng, theta, h, q, d, dev = _setup(13 + n_fc, H, V, max(DH, 1), n_fc, N)
    lam = 0.6
    adv, ce, g = T.gen_grad(theta, h, q, d, lam)
    D = K.Discriminator(dev(theta["w_lin"]), [dev(w) for w in theta["w_fc"]], [dev(b) for b in theta["b_fc"]], fc_hidden=DH)
    loss = torch.zeros(2, device="cuda")
    grad = torch.zeros(N, V, device="cuda")
    D.gen_grad(dev(h), dev(q), dev(d), lam, loss, grad)
    torch.cuda.synchronize()
    assert abs(loss[0].item() - adv) < TOL * abs(adv) and abs(loss[1].item() - ce) < TOL * abs(ce)
    _close(grad.cpu().numpy(), g, "dL_G/dd")
    # lambda = 0: the gradient is the distillation term's alone, (softmax(d) - softmax(q)) / N
    D.gen_grad(dev(h), dev(q), dev(d), 0.0, loss, grad)
    torch.cuda.synchronize()
    sm = lambda x: np.exp(x - x.max(-1, keepdims=True)) / np.exp(x - x.max(-1, keepdims=True)).sum(-1, keepdims=True)
    assert loss[0].item() == 0.0
    _close(grad.cpu().numpy(), (sm(d) - sm(q)) / N, "distillation gradient")


@pytest.mark.parametrize("Kb", [1, 2, 3])
def test_medusa_head_forward_and_update_match_oracle(Kb):
    import torch
    import paper_2408_08146_amd as K
    H, V, N = 200, 1000, 37
    rng, theta, h, q, _, dev = _setup(23 + Kb, H, V, 150, 2, N)
    blocks = [rng.normal(size=(H, H)) * 0.05 for _ in range(Kb)]
    w_lm = rng.normal(size=(V, H)) * 0.1
    lam, lr = 0.5, 0.2
    d_ref, _ = T.medusa_head_forward(blocks, w_lm, h)
    _, _, g = T.gen_grad(theta, h, q, d_ref, lam)
    new, grads = T.medusa_head_step(blocks, w_lm, h, g, lr)
    dblocks = [dev(b) for b in blocks]
    head = K.MedusaHeadTrainer(dblocks, dev(w_lm))
    D = K.Discriminator(dev(theta["w_lin"]), [dev(w) for w in theta["w_fc"]], [dev(b) for b in theta["b_fc"]], fc_hidden=150)
    d = torch.zeros(N, V, device="cuda")
    head.forward(dev(h), d)
    torch.cuda.synchronize()
    _close(d.cpu().numpy(), d_ref, "head logits")
    loss = torch.zeros(2, device="cuda")
    grad = torch.zeros(N, V, device="cuda")
    D.gen_grad(dev(h), dev(q), d, lam, loss, grad)          # the whole draft-head step of Algorithm 1 on the device
    head.step(dev(h), grad, lr)
    torch.cuda.synchronize()
    for k in range(Kb):
        _close(dblocks[k].cpu().numpy() - blocks[k].astype(np.float32), -lr * grads[k], f"block {k} update")


def test_training_argument_errors():
    import torch
    import paper_2408_08146_amd as K
    rng, theta, h, q, d, dev = _setup(1, 64, 100, 32, 2, 8)
    D = K.Discriminator(dev(theta["w_lin"]), [dev(w) for w in theta["w_fc"]], [dev(b) for b in theta["b_fc"]], fc_hidden=32)
    loss = torch.zeros(1, device="cuda")
    with pytest.raises(K.KoalaError):
        D.step(dev(h), dev(q), dev(d), -1.0, loss)            # negative step size
    D.shape.n_fc = 4
    with pytest.raises(K.KoalaError):
        D.step(dev(h), dev(q), dev(d), 0.1, loss)             # at most three fully connected layers
