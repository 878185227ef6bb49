"""Adversarial training step of a draft head (oracle; test infrastructure only).

Section 3.2 trains the draft head G against a discriminator D: D sees the target model's last
hidden state together with a row of token logits and estimates the probability that the logits
are the target's (and not the draft head's).  Algorithm 1 alternates a draft-head step on

    L_G = -lambda * E[log D(d)] + L_Distill(d, q)                                    (Eq. 5)

with a discriminator step on

    L_D = -E[log(1 - D(d))] - E[log D(q)]                                            (Eq. 6)

where d are the draft head's logits and q the target's for the same positions.

What the paper leaves open and this oracle (and the library) reads as follows:
  * D = Linear followed by fully connected layers: z = W_lin h maps the hidden state to the
    dimension of the logits, u = z + logits joins the two (same dimension, hence a sum), then n_fc
    fully connected layers with biases, ReLU between them, the last one of width 1, and a sigmoid.
    n_fc is the discriminator's layer count, which section 3.2 sets equal to the draft head's K;
  * an expectation is the mean over the positions of the batch; D's argument is the logits row
    itself (a sampled token would cut the gradient path to G);
  * L_Distill is the cross-entropy of softmax(d) against softmax(q) ("such as cross-entropy"),
    mean over positions;
  * the parameter update is plain gradient descent with step size lr (no optimiser is named).

Everything is written out layer by layer, forward and backward, in float64; the backward
formulas are pinned by finite differences of the forward ones in tests/test_oracle_train.py.
"""
from __future__ import annotations

import numpy as np


def _softplus(x):
    """log(1 + exp(x)) without overflow."""
    return np.maximum(x, 0.0) + np.log1p(np.exp(-np.abs(x)))


def _log_softmax(x):
    m = np.max(x, axis=-1, keepdims=True)
    return x - m - np.log(np.sum(np.exp(x - m), axis=-1, keepdims=True))


def disc_params(rng, hidden, vocab, fc_hidden, n_fc, std=0.02):
    """Random discriminator parameters: dict(w_lin [V,H], w_fc [list of n_fc matrices], b_fc [list])."""
    dims = [vocab] + [fc_hidden] * (n_fc - 1) + [1]
    return dict(w_lin=rng.normal(size=(vocab, hidden)) * std,
                w_fc=[rng.normal(size=(dims[i + 1], dims[i])) * std for i in range(n_fc)],
                b_fc=[rng.normal(size=(dims[i + 1],)) * std for i in range(n_fc)])


def disc_forward(theta, h, logits):
    """s = pre-sigmoid score of every row: D = sigmoid(s).  Returns (s [N], cache for the backward pass)."""
    z = h @ theta["w_lin"].T
    a = [z + logits]                                        # a[0] = u, a[k] = input of FC layer k
    pre = []
    n_fc = len(theta["w_fc"])
    for k in range(n_fc):
        y = a[k] @ theta["w_fc"][k].T + theta["b_fc"][k]
        pre.append(y)
        if k + 1 < n_fc:
            a.append(np.maximum(y, 0.0))
    return pre[-1][:, 0], dict(a=a, pre=pre)


def disc_backward(theta, h, cache, ds):
    """Given ds = dL/ds per row: gradients of all parameters and of u (the rows joined to z)."""
    n_fc = len(theta["w_fc"])
    g = ds[:, None]                                          # dL/d(pre of last layer)
    gw, gb = [None] * n_fc, [None] * n_fc
    for k in range(n_fc - 1, -1, -1):
        gw[k] = g.T @ cache["a"][k]
        gb[k] = g.sum(0)
        g = g @ theta["w_fc"][k]                             # dL/d a[k]
        if k > 0:
            g = g * (cache["pre"][k - 1] > 0.0)
    return dict(w_fc=gw, b_fc=gb, u=g)


def loss_d(theta, h, q, d):
    """Eq. 6 with means over the batch."""
    sd, _ = disc_forward(theta, h, d)
    sq, _ = disc_forward(theta, h, q)
    return float(np.mean(_softplus(sd)) + np.mean(_softplus(-sq)))      # -log(1-sigmoid(sd)) - log sigmoid(sq)


def disc_step(theta, h, q, d, lr):
    """One discriminator step (Algorithm 1): returns (L_D before the update, updated parameters)."""
    n = h.shape[0]
    sd, cd = disc_forward(theta, h, d)
    sq, cq = disc_forward(theta, h, q)
    loss = float(np.mean(_softplus(sd)) + np.mean(_softplus(-sq)))
    sig = lambda x: 1.0 / (1.0 + np.exp(-x))
    bd = disc_backward(theta, h, cd, sig(sd) / n)            # d/ds softplus(s) = sigmoid(s)
    bq = disc_backward(theta, h, cq, -(1.0 - sig(sq)) / n)   # d/ds softplus(-s) = -(1 - sigmoid(s))
    g_lin = (bd["u"] + bq["u"]).T @ h                        # u = W_lin h + logits
    new = dict(w_lin=theta["w_lin"] - lr * g_lin,
               w_fc=[w - lr * (a + b) for w, a, b in zip(theta["w_fc"], bd["w_fc"], bq["w_fc"])],
               b_fc=[w - lr * (a + b) for w, a, b in zip(theta["b_fc"], bd["b_fc"], bq["b_fc"])])
    grads = dict(w_lin=g_lin, w_fc=[a + b for a, b in zip(bd["w_fc"], bq["w_fc"])],
                 b_fc=[a + b for a, b in zip(bd["b_fc"], bq["b_fc"])])
    return loss, new, grads


def loss_g(theta, h, q, d, lam):
    """Eq. 5: (adversarial term, distillation term)."""
    sd, _ = disc_forward(theta, h, d)
    adv = lam * float(np.mean(_softplus(-sd)))               # -lambda * mean log sigmoid(sd)
    pq = np.exp(_log_softmax(q))
    ce = float(np.mean(-np.sum(pq * _log_softmax(d), axis=-1)))
    return adv, ce


def gen_grad(theta, h, q, d, lam):
    """Draft-head side of Algorithm 1 at the logits: (adversarial term, distillation term, dL_G/dd)."""
    n = h.shape[0]
    sd, cd = disc_forward(theta, h, d)
    adv = lam * float(np.mean(_softplus(-sd)))
    ls = _log_softmax(d)
    pq = np.exp(_log_softmax(q))
    ce = float(np.mean(-np.sum(pq * ls, axis=-1)))
    sig = 1.0 / (1.0 + np.exp(-sd))
    g_adv = disc_backward(theta, h, cd, -lam * (1.0 - sig) / n)["u"]     # du/dd = identity
    g_ce = (np.exp(ls) - pq) / n
    return adv, ce, g_adv + g_ce


def silu(x):
    return x / (1.0 + np.exp(-x))


def silu_grad(x):
    s = 1.0 / (1.0 + np.exp(-x))
    return s * (1.0 + x * (1.0 - s))


def medusa_head_forward(blocks, w_lm, h):
    """Medusa-style head of section 3.1: K residual blocks x <- x + SiLU(W x), then the LM head."""
    xs, ys = [h], []
    for w in blocks:
        y = xs[-1] @ w.T
        ys.append(y)
        xs.append(xs[-1] + silu(y))
    return xs[-1] @ w_lm.T, dict(xs=xs, ys=ys)


def medusa_head_step(blocks, w_lm, h, grad_d, lr):
    """Backward pass of the head for dL/dd = grad_d and one gradient-descent update of its blocks
    (the LM head is the target's and stays fixed).  Returns (updated blocks, their gradients)."""
    _, c = medusa_head_forward(blocks, w_lm, h)
    gx = grad_d @ w_lm
    grads = [None] * len(blocks)
    for k in range(len(blocks) - 1, -1, -1):
        gy = gx * silu_grad(c["ys"][k])
        grads[k] = gy.T @ c["xs"][k]
        gx = gx + gy @ blocks[k]
    return [w - lr * g for w, g in zip(blocks, grads)], grads
