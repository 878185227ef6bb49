"""Non-greedy (temperature) drafting and acceptance (oracle; test infrastructure only).

Section 2.2 states the rule for a chain of drafted tokens: token i, drawn from the draft
distribution d_i, is kept with probability min(1, q_i(x)/d_i(x)); at the first rejection a
replacement is drawn from norm(max(0, q - d)) and the rest is dropped; if everything is kept, one
more token is drawn from the target's next distribution.  Section 4.4 evaluates it at
temperature 1.

The paper does not say how this extends to a candidate tree.  The reading used here (and by the
library) is the multi-round form of the same rule: the k children of a node are k draws without
replacement from the node's draft distribution (draw order = child rank), and they are tried in
that order; after each rejection the target distribution is replaced by its normalised positive
part minus the draft distribution, and the rejected token is removed from the draft distribution,
which is renormalised.  On a chain template this is exactly the rule of section 2.2, and the tokens
it emits are distributed as the target's own samples.

Every random number is an input (uniforms in [0, 1)), so the device path can be given the same
ones.
"""
from __future__ import annotations

import numpy as np

from .tree import tree_depths, ancestor_mask, children_lists, expanded_nodes
from .spec import _w, eagle_rows


def softmax_t(logits, temperature=1.0):
    """softmax(logits / temperature) in fp64."""
    z = np.asarray(logits, np.float64) / float(temperature)
    e = np.exp(z - np.max(z))
    return e / np.sum(e)


def inverse_cdf(p, u):
    """Index of the first element at which the running sum of the (unnormalised, non-negative)
    weights p exceeds u * sum(p); the last positive element if rounding leaves none; 0 if no
    element is positive (a distribution that has been drawn empty)."""
    p = np.asarray(p, np.float64)
    c = np.cumsum(p)
    hit = np.nonzero(c > u * c[-1])[0]
    if len(hit):
        return int(hit[0])
    pos = np.nonzero(p > 0)[0]
    return int(pos[-1]) if len(pos) else 0


def draw_without_replacement(d, uniforms):
    """len(uniforms) draws from distribution d, each from what is left of d after the earlier
    draws were removed (renormalised).  Returns the drawn indices in draw order."""
    d = np.array(d, np.float64)
    out = []
    for u in uniforms:
        i = inverse_cdf(d, u)
        out.append(i)
        d[i] = 0.0
    return out


def accept_sample(tree_tokens, parent, rank, q_rows, d_rows, u_accept, u_resample):
    """Stochastic acceptance walk.  q_rows[i] / d_rows[i]: target / draft distribution over the
    vocabulary at node i (d_rows[i] is only read for nodes that have children); the children of
    a node are tried in rank order (the order they were drawn in); u_accept[c] decides child c,
    u_resample[i] draws the replacement (or bonus) token when the walk stops at node i.
    Returns (a, path, next_token) like the greedy walk."""
    ch = [sorted(k, key=lambda c: rank[c]) for k in children_lists(parent)]
    cur, path = 0, [0]
    while True:
        q = np.array(q_rows[cur], np.float64)
        if not ch[cur]:
            return len(path) - 1, path, inverse_cdf(q, u_resample[cur])       # bonus token from q
        d = np.array(d_rows[cur], np.float64)
        d = d / d.sum()
        q = q / q.sum()
        moved = False
        for c in ch[cur]:
            x = int(tree_tokens[c])
            if d[x] > 0 and u_accept[c] < min(1.0, q[x] / d[x]):
                cur = c
                path.append(c)
                moved = True
                break
            r = np.maximum(0.0, q - d)
            q = r / r.sum() if r.sum() > 0 else q
            d[x] = 0.0
            if d.sum() > 0:
                d = d / d.sum()
        if not moved:
            return len(path) - 1, path, inverse_cdf(q, u_resample[cur])       # from the residual


def eagle_expand_sample(cfg, Wt, Wd, dcache, C, feat_in, tok_in, parent, rank, u_draw, temperature=1.0,
                        dt=np.float64):
    """EAGLE-style draft with sampled children (Eq. 2 with x ~ d): as `eagle_expand`, but the
    children of node u are draws without replacement from softmax(draft logits at u / temperature)
    with uniforms u_draw[child], child rank = draw order.
    Returns dict(tokens[T], logits{u: [V]} for nodes with children)."""
    tok_in = np.asarray(tok_in)
    feat_in = np.asarray(feat_in, dt)
    T, m = len(parent), len(tok_in)
    depth = tree_depths(parent)
    mask = ancestor_mask(parent)
    ch = children_lists(parent)
    exp = expanded_nodes(parent)
    Cd = C - m
    lm = _w(Wt, "lm_head", dt)
    pos = [Cd + i for i in range(m)]
    f = eagle_rows(cfg, Wt, Wd, dcache, tok_in, feat_in, pos, pos, [range(Cd + i + 1) for i in range(m)], dt)
    f_hat = {0: f[m - 1]}
    logits = {0: lm @ f[m - 1]}
    slot = {u: C + e for e, u in enumerate(x for x in exp if x != 0)}
    tokens = np.zeros(T, np.int32)
    tokens[0] = tok_in[m - 1]
    D = int(depth.max()) if T > 1 else 0
    for d_ in range(D):
        level = [u for u in exp if depth[u] == d_]
        if d_ > 0 and level:
            vis = [list(range(C)) + [slot[v] for v in range(1, T) if mask[u, v]] for u in level]
            f = eagle_rows(cfg, Wt, Wd, dcache, [tokens[u] for u in level],
                           np.stack([f_hat[parent[u]] for u in level]),
                           [C - 1 + d_] * len(level), [slot[u] for u in level], vis, dt)
            for i, u in enumerate(level):
                f_hat[u] = f[i]
                logits[u] = lm @ f[i]
        for u in level:
            kids = sorted(ch[u], key=lambda c: rank[c])           # draw order
            draws = draw_without_replacement(softmax_t(logits[u], temperature), [u_draw[c] for c in kids])
            for c, x in zip(kids, draws):
                tokens[c] = x
    return dict(tokens=tokens, logits=logits)


def generate_sampled(cfg, Wt, Wd, prompt, n_new, parent, rank, uniforms, temperature=1.0, dt=np.float64):
    """Non-greedy generation loop (section 2.2 repeated; section 4.4 evaluates both kinds of head): prefill,
    then repeat sampled draft -> verify -> stochastic acceptance -> commit until n_new tokens exist (the
    first is drawn from the prefill's last distribution with uniforms[0][2][0]).  cfg["draft"] selects the
    head: "eagle" (Wd = its weights; the accepted path's features and tokens are its next catch-up rows) or
    "medusa" (Wd = the heads' blocks; only the newest feature is used).  uniforms[i] = (u_draw[T],
    u_accept[T], u_resample[T]) of iteration i.  Returns dict(tokens, accept_lens, C)."""
    from .spec import prefill, verify_tree, commit_path
    from .llama import KVCache
    T = len(parent)
    medusa = cfg.get("draft", "eagle") == "medusa"
    D = int(tree_depths(parent).max()) if T > 1 else 0
    cap = len(prompt) + n_new + 2 * T + 2
    tcache = KVCache(cfg["n_layers"], cfg["n_heads"], cap, cfg["head_dim"], dt)
    dcache = None if medusa else KVCache(cfg["K"], cfg["n_heads"], cap, cfg["head_dim"], dt)
    feats, logits = prefill(cfg, Wt, tcache, prompt, dt)
    root = inverse_cdf(softmax_t(logits[-1], temperature), uniforms[0][2][0])
    out, accept_lens = [root], []
    C = len(prompt)
    feat_in, tok_in = feats, np.asarray(list(prompt[1:]) + [root], np.int32)
    it = 0
    while len(out) < n_new:
        u_draw, u_acc, u_res = uniforms[it]
        if medusa:
            dr = medusa_expand_sample(cfg, Wt, Wd, feat_in[-1], int(tok_in[-1]), parent, rank, D, u_draw, temperature, dt)
        else:
            dr = eagle_expand_sample(cfg, Wt, Wd, dcache, C, feat_in, tok_in, parent, rank, u_draw, temperature, dt)
        tokens = dr["tokens"]
        feat, tl, _ = verify_tree(cfg, Wt, tcache, C, tokens, parent, dt)
        q = {i: softmax_t(tl[i], temperature) for i in range(T)}
        d = {u: softmax_t(row, temperature) for u, row in dr["logits"].items()}
        a, path, nxt = accept_sample(tokens, parent, rank, q, d, u_acc, u_res)
        C = commit_path(tcache, C, path)
        emitted = [int(tokens[p]) for p in path[1:]] + [nxt]
        out += emitted
        accept_lens.append(a)
        feat_in, tok_in = feat[path], np.asarray(emitted, np.int32)
        it += 1
    return dict(tokens=out[:n_new], accept_lens=accept_lens, C=C)


def medusa_expand_sample(cfg, Wt, Wm, feat_last, root_token, parent, rank, n_heads_used, u_draw, temperature=1.0,
                         dt=np.float64):
    """Medusa-style draft with sampled children: head j (one per depth, K residual blocks, shared
    LM head; section 3.1) gives one distribution for all nodes of depth j; the children of every
    node of depth j-1 are draws without replacement from it, each parent with the uniforms of its
    own children (draw order = rank).  Returns dict(tokens[T], logits{u: [V]} for nodes with
    children: the logits of the head that drafts u's children)."""
    from .llama import silu
    T = len(parent)
    depth = tree_depths(parent)
    ch = children_lists(parent)
    lm = _w(Wt, "lm_head", dt)
    head_logits = []
    for j in range(n_heads_used):
        x = np.asarray(feat_last, dt)
        for k in range(cfg["K"]):
            x = x + silu(_w(Wm, f"medusa.{j}.{k}", dt) @ x)
        head_logits.append(lm @ x)
    tokens = np.zeros(T, np.int32)
    tokens[0] = root_token
    logits = {}
    for u in range(T):                                   # parents precede children
        if not ch[u]:
            continue
        logits[u] = head_logits[int(depth[u])]
        kids = sorted(ch[u], key=lambda c: rank[c])
        draws = draw_without_replacement(softmax_t(logits[u], temperature), [u_draw[c] for c in kids])
        for c, x in zip(kids, draws):
            tokens[c] = x
    return dict(tokens=tokens, logits=logits)
