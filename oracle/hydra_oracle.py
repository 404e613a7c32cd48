"""CPU oracle for one step of Hydra decoding.  TEST INFRASTRUCTURE ONLY.

Only tests/, the smoke check and the benchmark's cpu_baseline leg may import
this file.  It shares no code with the HIP library and never calls it.  It is a
plain, slow, float64 numpy statement of what the hot path computes:

  * the frozen base model is a LLaMA-family decoder (paper, section 5 "Models"):
    pre-norm RMSNorm, rotary positions, multi-head attention, SwiGLU FFN,
    untied input embedding E and LM head, no biases;
  * plain greedy autoregressive decoding (paper, section 1) processes one token
    at a time against a flat KV cache:              `ar_*` functions;
  * a Hydra decoding step (paper, sections 2 "Tree decoding" and 3) is
      draft   -> `draft_tree`      heads f_Hydra,i(h_{t-1}, x_t, x^_{t+1..t+i-1}),
      verify  -> `tree_verify`     one base forward over the packed tree with
                                   an ancestors-only attention mask,
      accept  -> `accept_greedy`   candidate accepted iff it equals the base
                                   model's most likely token (section 2),
      compact -> `kv_compact`      keep the accepted tokens, discard the rest.

State carried between steps is the paper's (x_{<=t}, h_{t-1}): the KV cache
holds x_{<=t-1} (L tokens), `h_last` is the final hidden state (after the last
RMSNorm) of the most recently processed token, and `root` = x_t is the base
model's greedy token that has been emitted but not yet processed.

Weights arrive through a mapping name -> array (see synth.weights for names);
every array is converted to float64 when it is read, so a bf16 configuration is
"bf16-rounded weights, exact arithmetic".

Readings of points the paper leaves open are listed with the functions that
take them.  Nothing here is blocked, fused or reordered.
"""
from __future__ import annotations

import numpy as np


# ----------------------------------------------------------------------------
# tree bookkeeping (paper, section 2 "Tree decoding": nodes are candidate
# tokens, a root-to-node path is a candidate continuation)
# ----------------------------------------------------------------------------
class Tree:
    """Static topology given as a parent list with parent[n] < n, parent[0] = -1.

    Node 0 is the root x_t.  Children of a node keep the order in which they
    appear in the list; that order is their rank (rank 0 = most likely).
    """

    def __init__(self, parent):
        self.parent = [int(p) for p in parent]
        self.T = len(self.parent)
        assert self.T >= 1 and self.parent[0] == -1
        self.depth = [0] * self.T
        self.children = [[] for _ in range(self.T)]
        for n in range(1, self.T):
            p = self.parent[n]
            assert 0 <= p < n
            self.depth[n] = self.depth[p] + 1
            self.children[p].append(n)
        self.max_depth = max(self.depth)

    def path(self, n):
        """Nodes from the root down to n, both included."""
        out = []
        while n >= 0:
            out.append(n)
            n = self.parent[n]
        return out[::-1]


# ----------------------------------------------------------------------------
# elementwise pieces of the LLaMA-family decoder
# ----------------------------------------------------------------------------
def rmsnorm(x, g, eps):
    """x * g / sqrt(mean(x^2) + eps) over the last axis."""
    x = np.asarray(x, dtype=np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(g, dtype=np.float64)


def silu(x):
    x = np.asarray(x, dtype=np.float64)
    return x / (1.0 + np.exp(-x))


def rope(x, pos, theta):
    """Rotary embedding of a vector (or [..., Dh] array) at integer position pos.

    Reading: the LLaMA pairing of dimension j with j + Dh/2, frequency
    theta^(-2j/Dh), j = 0..Dh/2-1; position 0 is the identity.
    """
    x = np.asarray(x, dtype=np.float64)
    Dh = x.shape[-1]
    half = Dh // 2
    j = np.arange(half, dtype=np.float64)
    ang = float(pos) * theta ** (-2.0 * j / Dh)
    c, s = np.cos(ang), np.sin(ang)
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def softmax(s):
    s = np.asarray(s, dtype=np.float64)
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=-1, keepdims=True)


def top_k_ids(logits, k):
    """The k largest entries, ordered by (value descending, id ascending).

    Paper, section 2: a node with m children takes the m most likely tokens,
    sorted by descending probability.  Reading for ties: lowest id first.
    """
    logits = np.asarray(logits, dtype=np.float64)
    order = np.lexsort((np.arange(logits.shape[0]), -logits))
    return [int(t) for t in order[:k]]


def argmax_lowest(logits):
    """Most likely token; ties go to the lowest id."""
    return int(np.argmax(np.asarray(logits, dtype=np.float64)))


# ----------------------------------------------------------------------------
# model container
# ----------------------------------------------------------------------------
class Model:
    """Shape + weight lookup.  `weights[name]` may be numpy, torch or anything
    np.asarray understands after `.float()`; it is read as float64 each time."""

    def __init__(self, d, NL, H, Dh, F, V, K, mlp_layers, weights,
                 rms_eps=1e-6, rope_theta=10000.0, include_root_embedding=1,
                 keep_converted=False, medusa=0):
        self.d, self.NL, self.H, self.Dh, self.F, self.V = d, NL, H, Dh, F, V
        self.K, self.mlp_layers = K, mlp_layers
        self.eps, self.theta = rms_eps, rope_theta
        self.include_root_embedding = include_root_embedding
        self.medusa = medusa                          # 1: sequentially independent draft heads (paper, section 2)
        self.weights = weights
        self._kept = {} if keep_converted else None   # small models: convert once
        assert H * Dh == d

    def w(self, name):
        if self._kept is not None and name in self._kept:
            return self._kept[name]
        a = self.weights[name]
        if hasattr(a, "detach"):                      # torch tensor (any float dtype)
            a = a.detach().to("cpu").double().numpy()
        a = np.asarray(a, dtype=np.float64)
        if self._kept is not None:
            self._kept[name] = a
        return a


class FlatCache:
    """Per-sequence KV cache: K[l], V[l] of shape [capacity, H, Dh], float64."""

    def __init__(self, model, capacity):
        self.K = np.zeros((model.NL, capacity, model.H, model.Dh))
        self.V = np.zeros((model.NL, capacity, model.H, model.Dh))
        self.capacity = capacity


# ----------------------------------------------------------------------------
# plain autoregressive decoding: one token at a time (paper, section 1)
# ----------------------------------------------------------------------------
def ar_forward_token(model, cache, token, pos):
    """Process ONE token at position pos (cache holds positions 0..pos-1).

    Returns (hidden after the final RMSNorm [d], logits [V]) and stores the
    token's K/V at slot pos.  Written per token and per head on purpose: this
    is the definition the tree-masked forward is judged against.
    """
    m = model
    x = m.w("embed")[token].copy()
    for l in range(m.NL):
        p = f"layers.{l}."
        n1 = rmsnorm(x, m.w(p + "attn_norm"), m.eps)
        q = (m.w(p + "wq") @ n1).reshape(m.H, m.Dh)
        k = (m.w(p + "wk") @ n1).reshape(m.H, m.Dh)
        v = (m.w(p + "wv") @ n1).reshape(m.H, m.Dh)
        q = rope(q, pos, m.theta)
        k = rope(k, pos, m.theta)
        cache.K[l, pos] = k
        cache.V[l, pos] = v
        att = np.zeros((m.H, m.Dh))
        for h in range(m.H):
            keys = cache.K[l, :pos + 1, h]                    # [pos+1, Dh]
            vals = cache.V[l, :pos + 1, h]
            s = keys @ q[h] / np.sqrt(m.Dh)
            att[h] = softmax(s) @ vals
        a = x + m.w(p + "wo") @ att.reshape(m.d)
        n2 = rmsnorm(a, m.w(p + "ffn_norm"), m.eps)
        gate = m.w(p + "w_gate") @ n2
        up = m.w(p + "w_up") @ n2
        x = a + m.w(p + "w_down") @ (silu(gate) * up)
    h = rmsnorm(x, m.w("final_norm"), m.eps)
    return h, m.w("lm_head") @ h


def ar_prefill(model, cache, prompt):
    """Feed the prompt token by token.  Returns (L, h_last, root, last logits)."""
    h = logits = None
    for pos, tok in enumerate(prompt):
        h, logits = ar_forward_token(model, cache, int(tok), pos)
    return len(prompt), h, argmax_lowest(logits), logits


def ar_generate(model, prompt, n_new, capacity=None):
    """Plain greedy decoding: the first n_new generated tokens."""
    cache = FlatCache(model, capacity or (len(prompt) + n_new + 1))
    L, h, nxt, _ = ar_prefill(model, cache, prompt)
    out = []
    while len(out) < n_new:
        out.append(nxt)
        if len(out) == n_new:
            break
        h, logits = ar_forward_token(model, cache, nxt, L)
        L += 1
        nxt = argmax_lowest(logits)
    return out


# ----------------------------------------------------------------------------
# Hydra step, part 1: draft heads fill the candidate tree (paper, section 3)
# ----------------------------------------------------------------------------
def head_logits(model, i, h_last, path_tokens):
    """Draft logits of head i for one node.

    Paper, section 3: f_Hydra,i(h_{t-1}, x_t, x^_{t+1}, ..., x^_{t+i-1}) is an MLP
    on the hidden state concatenated, along the feature axis, with the input
    embeddings of x_t and of the earlier candidate tokens.  `path_tokens` are
    the i tokens on the root-to-node path (the root x_t first).
    Readings: hidden layer SiLU(W1 u + b1), no residual on it (widths differ);
    for Hydra++ (section 3.1, "Scaling") layers 2..n are z + SiLU(W z + b);
    a per-head vocabulary projection Wout without bias.  With
    include_root_embedding = 0 the embedding of x_t is left out of u.

    model.medusa (paper, section 2, "Lightweight heads as a draft model" and "Medusa
    decoding"): the head sees h_{t-1} only, p_draft = f_draft,i(h_{t-1}); it has one
    hidden layer with a skip connection around it, z = h + SiLU(W1 h + b1) with
    W1 [d, d]; the path tokens are ignored.
    """
    m = model
    if m.medusa:
        h = np.asarray(h_last, dtype=np.float64)
        z = h + silu(m.w(f"heads.{i}.w1") @ h + m.w(f"heads.{i}.b1"))
        for j in range(2, m.mlp_layers + 1):
            z = z + silu(m.w(f"heads.{i}.w{j}") @ z + m.w(f"heads.{i}.b{j}"))
        return m.w(f"heads.{i}.wout") @ z
    E = m.w("embed")
    toks = list(path_tokens)
    assert len(toks) == i
    if not m.include_root_embedding:
        toks = toks[1:]
    u = np.concatenate([np.asarray(h_last, dtype=np.float64)] + [E[t] for t in toks])
    z = silu(m.w(f"heads.{i}.w1") @ u + m.w(f"heads.{i}.b1"))
    for j in range(2, m.mlp_layers + 1):
        z = z + silu(m.w(f"heads.{i}.w{j}") @ z + m.w(f"heads.{i}.b{j}"))
    return m.w(f"heads.{i}.wout") @ z


def draft_tree(model, tree, h_last, root, forced_tokens=None):
    """Fill the tree: tok[0] = root; children of node n at depth i-1 are the
    top-(number of children) tokens of head i on n's path, best first.

    `forced_tokens` (tests only): tokens to assume on every path instead of the
    oracle's own picks, so a second implementation's choices can be audited
    node by node; the returned per-node logits then refer to those paths.
    Returns (tok [T], logits_of_expanded_nodes {n: [V]}).
    """
    assert tree.max_depth <= model.K, "tree deeper than the number of draft heads"
    tok = [0] * tree.T
    tok[0] = int(root)
    logits_at = {}
    for i in range(1, tree.max_depth + 1):
        for n in range(tree.T):
            if tree.depth[n] != i - 1 or not tree.children[n]:
                continue
            src = forced_tokens if forced_tokens is not None else tok
            ptoks = [int(src[a]) for a in tree.path(n)]
            ptoks[0] = int(root)
            lg = head_logits(model, i, h_last, ptoks)
            logits_at[n] = lg
            best = top_k_ids(lg, len(tree.children[n]))
            for c, t in zip(tree.children[n], best):
                tok[c] = t
    return tok, logits_at


# ----------------------------------------------------------------------------
# Hydra step, part 2: tree verification (paper, section 2 "Tree decoding")
# ----------------------------------------------------------------------------
def ancestor_mask(tree):
    """mask[n, a] = True iff a is n itself or an ancestor of n.

    Paper, section 2: each packed token may attend only to its parents in the
    tree.  Reading: all ancestors and the token itself, plus the whole verified
    prefix; nothing else makes the result equal sequential decoding.
    """
    mask = np.zeros((tree.T, tree.T), dtype=bool)
    for n in range(tree.T):
        for a in tree.path(n):
            mask[n, a] = True
    return mask


def tree_verify(model, cache, L, tree, tok):
    """One base forward over all T tree tokens at once.

    Node n sits at position L + depth[n]; its keys are cache slots 0..L-1 and
    the nodes allowed by `ancestor_mask`; its K/V are stored at slot L + n.
    Returns hidden [T,d] (after the final RMSNorm), logits [T,V], argmax [T].
    """
    m, T = model, tree.T
    assert L + T <= cache.capacity
    mask = ancestor_mask(tree)
    allowed = np.concatenate([np.ones((T, L), dtype=bool), mask], axis=1)   # [T, L+T]
    X = m.w("embed")[np.asarray(tok, dtype=np.int64)].copy()                 # [T, d]
    for l in range(m.NL):
        p = f"layers.{l}."
        N1 = rmsnorm(X, m.w(p + "attn_norm"), m.eps)
        Q = (N1 @ m.w(p + "wq").T).reshape(T, m.H, m.Dh)
        Kn = (N1 @ m.w(p + "wk").T).reshape(T, m.H, m.Dh)
        Vn = (N1 @ m.w(p + "wv").T).reshape(T, m.H, m.Dh)
        for n in range(T):
            Q[n] = rope(Q[n], L + tree.depth[n], m.theta)
            Kn[n] = rope(Kn[n], L + tree.depth[n], m.theta)
        cache.K[l, L:L + T] = Kn
        cache.V[l, L:L + T] = Vn
        A = np.zeros((T, m.H, m.Dh))
        for h in range(m.H):
            S = Q[:, h] @ cache.K[l, :L + T, h].T / np.sqrt(m.Dh)           # [T, L+T]
            S = np.where(allowed, S, -np.inf)
            A[:, h] = softmax(S) @ cache.V[l, :L + T, h]
        Y = X + A.reshape(T, m.d) @ m.w(p + "wo").T
        N2 = rmsnorm(Y, m.w(p + "ffn_norm"), m.eps)
        X = Y + (silu(N2 @ m.w(p + "w_gate").T) * (N2 @ m.w(p + "w_up").T)) @ m.w(p + "w_down").T
    Hid = rmsnorm(X, m.w("final_norm"), m.eps)
    logits = Hid @ m.w("lm_head").T
    return Hid, logits, [argmax_lowest(logits[n]) for n in range(T)]


def tree_attention(q, keys, vals, L, tree):
    """The attention of `tree_verify` alone, for one head.

    q [T,Dh] (already rotated), keys/vals [L+T,Dh] with node n at row L+n.
    """
    T = tree.T
    allowed = np.concatenate([np.ones((T, L), dtype=bool), ancestor_mask(tree)], axis=1)
    Dh = q.shape[-1]
    S = np.asarray(q, np.float64) @ np.asarray(keys, np.float64)[:L + T].T / np.sqrt(Dh)
    S = np.where(allowed, S, -np.inf)
    return softmax(S) @ np.asarray(vals, np.float64)[:L + T]


# ----------------------------------------------------------------------------
# Hydra step, parts 3 and 4: greedy acceptance and cache compaction
# ----------------------------------------------------------------------------
def accept_greedy(tree, tok, argmax):
    """Longest root path whose every candidate equals the base model's greedy
    token at its parent (paper, section 2, greedy acceptance).

    The root is x_t itself and always counts, so 1 <= n_acc <= max_depth + 1
    ("acceptance length = tokens generated per decoding step", section 5).
    If several children hold the matching token, the lowest node id is taken.
    Returns (n_acc, path, next_root, last_node).
    """
    cur, path = 0, [0]
    while True:
        g = int(argmax[cur])
        nxt = None
        for c in tree.children[cur]:
            if int(tok[c]) == g:
                nxt = c
                break
        if nxt is None:
            break
        cur = nxt
        path.append(cur)
    return len(path), path, int(argmax[cur]), cur


def kv_compact(cache, L, path):
    """Keep the accepted tokens: slot L + path[j] -> slot L + j, every layer.

    Paper, sections 1-2: the accepted subset is appended to the sequence, the
    rest discarded.  path[j] >= j, so ascending j never overwrites a source.
    Returns the new length.
    """
    for j, n in enumerate(path):
        if n != j:
            cache.K[:, L + j] = cache.K[:, L + n]
            cache.V[:, L + j] = cache.V[:, L + n]
    return L + len(path)


# ----------------------------------------------------------------------------
# Typical acceptance (paper, section 6.3): a candidate token x^ at node c, child
# of node p, passes if   p_base(x^ | path to p; tau) > min(eps, alpha * exp(-H))
# with p_base(. ; tau) = softmax(logits[p] / tau) and H its entropy (natural log).
#
# Readings (the paper gives the per-token test only): the accepted continuation is
# the deepest node all of whose path tokens pass, the lowest node id among equally
# deep ones; the root x_t always counts; the next root is drawn from
# p_base(. | accepted path; tau) by inverting its cumulative distribution in token
# id order at a uniform number u in [0, 1) supplied by the caller (u = None: the
# most likely token, lowest id at ties).
# ----------------------------------------------------------------------------
def tempered_probs(logits_row, tau):
    z = np.asarray(logits_row, dtype=np.float64) / tau
    return softmax(z)


def entropy(p):
    p = np.asarray(p, dtype=np.float64)
    nz = p > 0
    return float(-np.sum(p[nz] * np.log(p[nz])))


def typical_pass(logits_row, token, tau, eps, alpha):
    """The per-token test of section 6.3 for a child carrying `token` under a node whose logits are given."""
    p = tempered_probs(logits_row, tau)
    return bool(p[int(token)] > min(eps, alpha * np.exp(-entropy(p))))


def sample_inverse_cdf(p, u):
    """Smallest id v with p[0] + ... + p[v] > u * sum(p)."""
    c = np.cumsum(np.asarray(p, dtype=np.float64))
    v = int(np.searchsorted(c, u * c[-1], side="right"))
    return min(v, len(c) - 1)


def accept_typical(tree, tok, logits, tau, eps, alpha, u=None):
    """Returns (n_acc, path, next_root, last_node) under the typical-acceptance criterion."""
    ok = [True] * tree.T
    for c in range(1, tree.T):
        ok[c] = typical_pass(logits[tree.parent[c]], tok[c], tau, eps, alpha)
    best = 0
    reach = [False] * tree.T
    reach[0] = True
    for c in range(1, tree.T):                                   # parents come before children
        reach[c] = reach[tree.parent[c]] and ok[c]
        if reach[c] and tree.depth[c] > tree.depth[best]:
            best = c                                             # first (lowest id) node of a new depth
    path = tree.path(best)
    if u is None:
        nxt = argmax_lowest(logits[best])
    else:
        nxt = sample_inverse_cdf(tempered_probs(logits[best], tau), u)
    return len(path), list(path), int(nxt), best


# ----------------------------------------------------------------------------
# Hydra++ prefix attention (paper, section 3.1 item 3; appendix, "Hydra-specific
# prefix attention"): one more decoder layer on top of the base model whose only
# role is to produce the hidden state the draft heads read.  It runs over the
# verified sequence with its own K/V and is queried once per decoding step; the
# heads take its representation of the last verified token in place of h_{t-1}.
#
# Readings (the paper does not fix them): the layer's input at position p is the
# base model's hidden state of token p as the LM head sees it (after the final
# RMSNorm); its output is the residual stream after the layer, with no further norm;
# it is an ordinary pre-norm Llama decoder layer (weights "prefix.*") with rotary
# positions 0, 1, 2, ...
# ----------------------------------------------------------------------------
class PrefixCache:
    """K/V of the prefix-attention layer: [capacity, H, Dh], float64."""

    def __init__(self, model, capacity):
        self.K = np.zeros((capacity, model.H, model.Dh))
        self.V = np.zeros((capacity, model.H, model.Dh))
        self.capacity = capacity


def prefix_token(model, pcache, x, pos):
    """The prefix-attention layer on ONE hidden state x [d] at position pos
    (pcache holds positions 0..pos-1).  Returns the layer's output [d]."""
    m = model
    x = np.asarray(x, dtype=np.float64)
    n1 = rmsnorm(x, m.w("prefix.attn_norm"), m.eps)
    q = rope((m.w("prefix.wq") @ n1).reshape(m.H, m.Dh), pos, m.theta)
    k = rope((m.w("prefix.wk") @ n1).reshape(m.H, m.Dh), pos, m.theta)
    pcache.K[pos] = k
    pcache.V[pos] = (m.w("prefix.wv") @ n1).reshape(m.H, m.Dh)
    att = np.zeros((m.H, m.Dh))
    for h in range(m.H):
        s = pcache.K[:pos + 1, h] @ q[h] / np.sqrt(m.Dh)
        att[h] = softmax(s) @ pcache.V[:pos + 1, h]
    a = x + m.w("prefix.wo") @ att.reshape(m.d)
    n2 = rmsnorm(a, m.w("prefix.ffn_norm"), m.eps)
    return a + m.w("prefix.w_down") @ (silu(m.w("prefix.w_gate") @ n2) * (m.w("prefix.w_up") @ n2))


def prefix_chunk(model, pcache, L, X):
    """The same layer on n consecutive hidden states X [n, d] at positions L..L+n-1
    in one causally masked pass (what a chunked implementation computes).  Must equal
    prefix_token applied one position at a time."""
    m = model
    X = np.asarray(X, dtype=np.float64)
    n = X.shape[0]
    N1 = rmsnorm(X, m.w("prefix.attn_norm"), m.eps)
    Q = (N1 @ m.w("prefix.wq").T).reshape(n, m.H, m.Dh)
    Kn = (N1 @ m.w("prefix.wk").T).reshape(n, m.H, m.Dh)
    for j in range(n):
        Q[j] = rope(Q[j], L + j, m.theta)
        Kn[j] = rope(Kn[j], L + j, m.theta)
    pcache.K[L:L + n] = Kn
    pcache.V[L:L + n] = (N1 @ m.w("prefix.wv").T).reshape(n, m.H, m.Dh)
    allowed = np.arange(L + n)[None, :] <= (L + np.arange(n))[:, None]
    A = np.zeros((n, m.H, m.Dh))
    for h in range(m.H):
        S = np.where(allowed, Q[:, h] @ pcache.K[:L + n, h].T / np.sqrt(m.Dh), -np.inf)
        A[:, h] = softmax(S) @ pcache.V[:L + n, h]
    Y = X + A.reshape(n, m.d) @ m.w("prefix.wo").T
    N2 = rmsnorm(Y, m.w("prefix.ffn_norm"), m.eps)
    return Y + (silu(N2 @ m.w("prefix.w_gate").T) * (N2 @ m.w("prefix.w_up").T)) @ m.w("prefix.w_down").T


def hydra_step(model, cache, tree, L, h_last, root, draft_hook=None, pcache=None, typical=None):
    """One full step.  Returns (emitted tokens, new L, new h_last, new root, info).

    With `pcache` (Hydra++ prefix attention) h_last is the prefix layer's output at the
    last verified token: after acceptance the layer is fed the base hidden states of the
    accepted tokens, one position each, and its last output becomes the new h_last.

    typical = None: greedy acceptance (section 2).  typical = (tau, eps, alpha, u): the typical
    acceptance criterion of section 6.3 decides the accepted path and the next root is the most
    likely token at its end (u None) or drawn there at the uniform number u (see accept_typical)."""
    tok, _ = draft_tree(model, tree, h_last, root)
    if draft_hook is not None:
        tok = draft_hook(tok)
    hidden, logits, amax = tree_verify(model, cache, L, tree, tok)
    if typical is None:
        n_acc, path, next_root, last = accept_greedy(tree, tok, amax)
    else:
        tau, eps, alpha, u = typical
        n_acc, path, next_root, last = accept_typical(tree, tok, logits, tau, eps, alpha, u)
    emitted = [int(tok[n]) for n in path]
    L2 = kv_compact(cache, L, path)
    info = {"tok": tok, "argmax": amax, "path": path, "n_acc": n_acc, "logits": logits, "hidden": hidden, "next_root": next_root}
    h_new = hidden[last]
    if pcache is not None:
        for j, n in enumerate(path):
            h_new = prefix_token(model, pcache, hidden[n], L + j)
    return emitted, L2, h_new, next_root, info


def hydra_generate(model, tree, prompt, n_new, draft_hook=None, capacity=None, prefix=False, typical=None, u_per_step=None,
                   step_log=None):
    """Hydra decoding: the first n_new generated tokens and the per-step acceptance lengths.
    Greedy acceptance unless typical = (tau, eps, alpha) is given (section 6.3); then step s draws its
    next root at u_per_step[s] (u_per_step None: the most likely token).  prefix=True: Hydra++ prefix
    attention.  step_log, if a list, receives every step's info dictionary."""
    cap = capacity or (len(prompt) + n_new + tree.T + tree.max_depth + 2)
    cache = FlatCache(model, cap)
    pcache = PrefixCache(model, cap) if prefix else None
    if prefix:
        h_last = logits = None
        for pos, t in enumerate(prompt):
            h, logits = ar_forward_token(model, cache, int(t), pos)
            h_last = prefix_token(model, pcache, h, pos)
        L, root = len(prompt), argmax_lowest(logits)
    else:
        L, h_last, root, _ = ar_prefill(model, cache, prompt)
    out, acc = [], []
    while len(out) < n_new:
        hook = (lambda t, _n=len(out): draft_hook(t, _n)) if draft_hook else None
        typ = None
        if typical is not None:
            typ = (typical[0], typical[1], typical[2], None if u_per_step is None else float(u_per_step[len(acc)]))
        emitted, L, h_last, root, info = hydra_step(model, cache, tree, L, h_last, root, hook, pcache, typ)
        out += emitted
        acc.append(info["n_acc"])
        if step_log is not None:
            step_log.append(info)
    return out[:n_new], acc
