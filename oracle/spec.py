"""One draft-then-verify iteration, step by step (oracle; test infrastructure only).

Notation follows the paper: the target model M_q (Eq. 1), the draft head M_d
producing candidate tokens (Eq. 2), parallel verification (Eq. 3), and the
greedy acceptance rule of section 4.1 (a drafted token is kept only if it
equals the target's greedy next token; the target's own token is appended
after the last kept one, section 2.2).

Conventions (the paper leaves them open; they are choices of this build):
  * committed tokens x_0..x_n; x_n (the newest, decided by the target but not
    yet run through it) is the tree root; the target cache holds x_0..x_{n-1},
    so its length is C = n;
  * the "feature" feat_i is the target's hidden state at position i *after* the
    final RMSNorm, i.e. exactly what the LM head consumes;
  * EAGLE-style draft row i pairs feat_i with the following token x_{i+1} and
    has position id i; its output predicts feat_{i+1};
  * node 0 of the tree is the root; a node of depth d sits at position C + d in
    the target and C - 1 + d in the draft.

`W*` arguments are weight providers: anything with `.f32(name) -> ndarray`
(or a plain dict).  `cfg` is a dict with hidden, n_heads, head_dim, ffn, vocab,
n_layers, rms_eps, rope_base (and K / medusa_heads for the draft).
"""
from __future__ import annotations

import numpy as np

from .llama import rmsnorm, silu, decoder_layer_rows, KVCache
from .tree import tree_depths, ancestor_mask, children_lists, expanded_nodes

_LAYER_KEYS = ("in_norm", "wq", "wk", "wv", "wo", "post_norm", "wgate", "wup", "wdown")


def _w(W, name, dt):
    a = W[name] if isinstance(W, dict) else W.f32(name)
    return np.asarray(a, dtype=dt)


def _layer(W, prefix, l, dt):
    return {k: _w(W, f"{prefix}layers.{l}.{k}", dt) for k in _LAYER_KEYS}


# ----------------------------------------------------------------------------
# target model
# ----------------------------------------------------------------------------
def target_rows(cfg, W, cache: KVCache, tokens, pos, slots, visible, dt=np.float64,
                n_layers=None):
    """Run the target on new rows (Eq. 1 / Eq. 3): x = E[token]; L decoder
    layers; feat = RMSNorm(x); logits = W_lm feat.  Returns (feat, logits)."""
    x = _w(W, "embed", dt)[np.asarray(tokens)]
    L = cfg["n_layers"] if n_layers is None else n_layers
    for l in range(L):
        x = decoder_layer_rows(x, pos, slots, visible, _layer(W, "", l, dt), cache.k[l], cache.v[l],
                               cfg["n_heads"], cfg["head_dim"], cfg["rms_eps"], cfg["rope_base"], cache.store)
    feat = rmsnorm(x, _w(W, "final_norm", dt), cfg["rms_eps"])
    logits = feat @ _w(W, "lm_head", dt).T
    return feat, logits


def decode_one(cfg, W, cache, C, token, dt=np.float64):
    """Plain autoregressive step (Eq. 1): feed `token` at position C; it sees
    rows 0..C.  Returns (feat[H], logits[V]); the caller sets C <- C + 1."""
    feat, logits = target_rows(cfg, W, cache, [token], [C], [C], [range(C + 1)], dt)
    return feat[0], logits[0]


def prefill(cfg, W, cache, tokens, dt=np.float64):
    """Feed tokens one at a time from an empty cache.  Returns feats[n,H], logits[n,V]."""
    fs, ls = [], []
    for i, t in enumerate(tokens):
        f, l = decode_one(cfg, W, cache, i, int(t), dt)
        fs.append(f)
        ls.append(l)
    return np.stack(fs), np.stack(ls)


def greedy_reference(cfg, W, prompt, n_new, dt=np.float64):
    """The first n_new tokens plain greedy decoding emits after `prompt` (Eq. 1 with argmax)."""
    cache = KVCache(cfg["n_layers"], cfg["n_heads"], len(prompt) + n_new + 1, cfg["head_dim"], dt)
    _, logits = prefill(cfg, W, cache, prompt, dt)
    out = [int(np.argmax(logits[-1]))]
    C = len(prompt)
    while len(out) < n_new:
        _, l = decode_one(cfg, W, cache, C, out[-1], dt)
        C += 1
        out.append(int(np.argmax(l)))
    return out


# ----------------------------------------------------------------------------
# verification of a candidate tree (Eq. 3) and greedy acceptance
# ----------------------------------------------------------------------------
def verify_tree(cfg, W, cache, C, tree_tokens, parent, dt=np.float64, n_layers=None):
    """All T nodes in one pass: node i has position C + depth(i), its key/value
    go to slot C + i, and it sees the C context rows plus itself and its
    ancestors.  Returns (feat[T,H], logits[T,V], greedy[T])."""
    T = len(parent)
    depth = tree_depths(parent)
    mask = ancestor_mask(parent)
    pos = [C + int(depth[i]) for i in range(T)]
    slots = [C + i for i in range(T)]
    visible = [list(range(C)) + [C + j for j in range(T) if mask[i, j]] for i in range(T)]
    feat, logits = target_rows(cfg, W, cache, tree_tokens, pos, slots, visible, dt, n_layers)
    greedy = np.argmax(logits, axis=-1).astype(np.int32)      # first maximum = lowest id
    return feat, logits, greedy


def accept_greedy(tree_tokens, greedy, parent):
    """Walk down from the root: step to the (lowest-index) child whose token is
    the target's greedy token at the current node; stop when none is.  Returns
    (a, path, next_token): a accepted drafted tokens, path = node ids root..last
    accepted (length a+1), next_token = the target's token after the path."""
    ch = children_lists(parent)
    cur, path = 0, [0]
    while True:
        nxt = [c for c in ch[cur] if int(tree_tokens[c]) == int(greedy[cur])]
        if not nxt:
            break
        cur = nxt[0]
        path.append(cur)
    return len(path) - 1, path, int(greedy[cur])


def commit_path(cache: KVCache, C, path, n_layers=None):
    """Make the accepted nodes context rows C..C+a (their rotary positions are
    already C + depth).  Returns the new context length."""
    L = len(cache.k) if n_layers is None else n_layers
    for l in range(L):
        for j, node in enumerate(path):
            cache.k[l][:, C + j, :] = cache.k[l][:, C + node, :]
            cache.v[l][:, C + j, :] = cache.v[l][:, C + node, :]
    return C + len(path)


def topk_desc(x, k):
    """Indices of the k largest entries, descending; equal values: lower index first."""
    return np.argsort(-x, kind="stable")[:k].astype(np.int32)


# ----------------------------------------------------------------------------
# EAGLE-style K-layer draft head (section 3.1)
# ----------------------------------------------------------------------------
def eagle_rows(cfg, Wt, Wd, dcache, tokens, feats, pos, slots, visible, dt=np.float64):
    """Embedding -> Linear over [embedding ; feature] -> K decoder layers.
    Returns the predicted next features f_hat[T,H] (no norm after the last layer)."""
    emb = _w(Wt, "embed", dt)[np.asarray(tokens)]
    z = np.concatenate([emb, np.asarray(feats, dt)], axis=-1)
    x = z @ _w(Wd, "draft.fc", dt).T
    for k in range(cfg["K"]):
        x = decoder_layer_rows(x, pos, slots, visible, _layer(Wd, "draft.", k, dt), dcache.k[k],
                               dcache.v[k], cfg["n_heads"], cfg["head_dim"], cfg["rms_eps"],
                               cfg["rope_base"], dcache.store)
    return x


def eagle_expand(cfg, Wt, Wd, dcache, C, feat_in, tok_in, parent, rank, topk, dt=np.float64):
    """Draft step (Eq. 2) for the autoregressive head, filling a static tree.

    feat_in[m,H], tok_in[m]: the m newest (feature, following token) pairs;
    tok_in[m-1] is the root.  The draft cache holds rows 0..C-m-1 on entry and
    rows 0..C-1 afterwards (tree rows beyond C are scratch).  Level by level,
    every node that has children in the template is run through the head (the
    root's row is catch-up row m-1); its logits' top-k, in rank order, become
    its children's tokens.  Returns dict(tokens[T], scores[T], f_hat{node},
    logits{node}).
    """
    m = len(tok_in)
    T = len(parent)
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
    scores = np.zeros(T, np.float64)
    tokens[0] = tok_in[m - 1]
    D = int(depth.max()) if T > 1 else 0
    for d in range(D):
        level = [u for u in exp if depth[u] == d]
        if d > 0 and level:
            vis = [list(range(C)) + [slot[v] for v in range(1, T) if mask[u, v]] for u in level]
            f = eagle_rows(cfg, Wt, Wd, dcache, [tokens[u] for u in level],
                           np.stack([f_hat[parent[u]] for u in level]),
                           [C - 1 + d] * len(level), [slot[u] for u in level], vis, dt)
            for i, u in enumerate(level):
                f_hat[u] = f[i]
                logits[u] = lm @ f[i]
        for u in level:
            top = topk_desc(logits[u], int(topk[d]))
            for c in ch[u]:
                tokens[c] = top[rank[c]]
                scores[c] = logits[u][tokens[c]]
    return dict(tokens=tokens, scores=scores, f_hat=f_hat, logits=logits)


# ----------------------------------------------------------------------------
# Medusa-style K-layer heads (section 3.1)
# ----------------------------------------------------------------------------
def medusa_expand(cfg, Wt, Wm, feat_last, root_token, parent, rank, topk, dt=np.float64):
    """Non-autoregressive draft (Eq. 2): head j (j = 1..D) applies K residual
    blocks x <- x + SiLU(W_{j,k} x) to the newest feature, the shared LM head
    maps the result to logits, and every depth-j node of rank r receives that
    head's rank-r token.  Returns dict(tokens[T], scores[T], logits[D,V])."""
    T = len(parent)
    depth = tree_depths(parent)
    lm = _w(Wt, "lm_head", dt)
    D = len(topk)
    head_logits = []
    for j in range(D):
        x = np.asarray(feat_last, dt)
        for k in range(cfg["K"]):
            x = x + silu(_w(Wm, f"medusa.{j}.{k}", dt) @ x)
        head_logits.append(lm @ x)
    tokens = np.zeros(T, np.int32)
    scores = np.zeros(T, np.float64)
    tokens[0] = root_token
    for i in range(1, T):
        j = int(depth[i]) - 1
        top = topk_desc(head_logits[j], int(topk[j]))
        tokens[i] = top[rank[i]]
        scores[i] = head_logits[j][tokens[i]]
    return dict(tokens=tokens, scores=scores, logits=np.stack(head_logits))


# ----------------------------------------------------------------------------
# whole iteration
# ----------------------------------------------------------------------------
def iteration_eagle(cfg, Wt, Wd, tcache, dcache, C, feat_in, tok_in, parent, rank, topk,
                    dt=np.float64, override_tokens=None):
    """draft -> verify -> accept -> commit.  `override_tokens(tokens)` lets a
    test replace drafted tokens before verification.  Returns a dict with the
    emitted tokens, the new context length and the next iteration's
    (feat_in, tok_in)."""
    dr = eagle_expand(cfg, Wt, Wd, dcache, C, feat_in, tok_in, parent, rank, topk, dt)
    tokens = dr["tokens"] if override_tokens is None else override_tokens(dr["tokens"].copy())
    feat, logits, greedy = verify_tree(cfg, Wt, tcache, C, tokens, parent, dt)
    a, path, nxt = accept_greedy(tokens, greedy, parent)
    C2 = commit_path(tcache, C, path)
    emitted = [int(tokens[p]) for p in path[1:]] + [nxt]
    return dict(tree_tokens=tokens, feat=feat, logits=logits, greedy=greedy, accept_len=a,
                path=path, next_token=nxt, emitted=emitted, C=C2,
                feat_in=feat[path], tok_in=np.asarray(emitted, np.int32), draft=dr)


# ----------------------------------------------------------------------------
# generation loop and its statistics (sections 2.2, 4.1)
# ----------------------------------------------------------------------------
def generate_speculative(cfg, Wt, Wd, prompt, n_new, parent, rank, topk, dt=np.float64):
    """Prefill `prompt` with the target, then repeat draft -> verify -> accept -> commit until
    at least n_new tokens were emitted (the first of them is the prefill's own greedy token).
    cfg["draft"] selects the head: "eagle" (the draft cache is brought up to date by the
    catch-up rows of every call, all prompt rows in the first) or "medusa".
    Returns dict(tokens[n_new], accept_lens[iterations], trees[iterations][T], C)."""
    T = len(parent)
    cap = len(prompt) + n_new + 2 * T + 2
    tcache = KVCache(cfg["n_layers"], cfg["n_heads"], cap, cfg["head_dim"], dt)
    feats, logits = prefill(cfg, Wt, tcache, prompt, dt)
    root = int(np.argmax(logits[-1]))
    out, accept_lens, trees = [root], [], []
    C = len(prompt)
    eagle = cfg["draft"] == "eagle"
    if eagle:
        dcache = KVCache(cfg["K"], cfg["n_heads"], cap, cfg["head_dim"], dt)
        feat_in, tok_in = feats, np.asarray(list(prompt[1:]) + [root], np.int32)
    else:
        feat_in, tok_in = feats[-1:], np.asarray([root], np.int32)
    while len(out) < n_new:
        if eagle:
            tokens = eagle_expand(cfg, Wt, Wd, dcache, C, feat_in, tok_in, parent, rank, topk, dt)["tokens"]
        else:
            tokens = medusa_expand(cfg, Wt, Wd, feat_in[-1], int(tok_in[-1]), parent, rank, topk, dt)["tokens"]
        feat, _, greedy = verify_tree(cfg, Wt, tcache, C, tokens, parent, dt)
        a, path, nxt = accept_greedy(tokens, greedy, parent)
        C = commit_path(tcache, C, path)
        emitted = [int(tokens[p]) for p in path[1:]] + [nxt]
        out += emitted
        accept_lens.append(a)
        trees.append(np.asarray(tokens).copy())
        feat_in, tok_in = feat[path], np.asarray(emitted, np.int32)
    return dict(tokens=out[:n_new], accept_lens=accept_lens, trees=trees, C=C)


def mean_tokens_per_iteration(accept_lens):
    """Average number of tokens one draft-verify iteration yields (section 4.1): every
    iteration emits its accepted drafted tokens plus the target's own next token."""
    return float(np.mean(np.asarray(accept_lens) + 1)) if len(accept_lens) else 0.0


def n_alpha(accept_lens, max_depth):
    """Acceptance rate of the n-th drafted token given that the n-1 before it were accepted
    (section 4.1), n = 1..max_depth, from the accepted lengths of chain drafts:
    alpha_n = #{iterations with a >= n} / #{iterations with a >= n-1}; nan where the
    denominator is zero."""
    a = np.asarray(accept_lens)
    out = []
    for n in range(1, max_depth + 1):
        den = int(np.sum(a >= n - 1))
        out.append(float(np.sum(a >= n)) / den if den else float("nan"))
    return out
