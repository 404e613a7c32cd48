"""Pins for the CPU oracle: what the paper and the mathematics fix.

None of these re-types the oracle's formulas.  Each compares the oracle with
something else: a library routine (HF LLaMA, torch SDPA), a closed form, an
invariant the paper states, or brute force on tiny inputs.

Citations: "tree = sequential" and the ancestor mask are section 2 ("Tree
decoding"); greedy speculative = greedy autoregressive is section 5
("Evaluation"); the head definition is section 3; the Medusa special case is
the displayed independence equation of section 3.
"""
import itertools

import numpy as np
import pytest
import torch

from oracle import hydra_oracle as O
from synth import chain_tree, frozen_tree, random_tree, star_tree, uniform_tokens
from helpers import make_weights, oracle_model, small_shape


# ------------------------------------------------------------------ library pins
# The library computes its RMSNorm and rotary tables in fp32 even in a float64
# model, so agreement stops near 1e-6 on logits of size 1..5; a structural slip
# (pairing, order, transposed operand, missing term) moves them by more than 1e-2.
_HF_TOL = 5e-6

def _hf_llama(cfg, weights):
    from transformers import LlamaConfig, LlamaForCausalLM
    hc = LlamaConfig(vocab_size=cfg.V, hidden_size=cfg.d, intermediate_size=cfg.F,
                     num_hidden_layers=cfg.NL, num_attention_heads=cfg.H, num_key_value_heads=cfg.H,
                     rms_norm_eps=cfg.rms_eps, rope_theta=cfg.rope_theta, max_position_embeddings=256,
                     tie_word_embeddings=False, attention_bias=False, mlp_bias=False, hidden_act="silu",
                     attn_implementation="eager")
    m = LlamaForCausalLM(hc).double().eval()
    sd = {"model.embed_tokens.weight": weights["embed"], "lm_head.weight": weights["lm_head"],
          "model.norm.weight": weights["final_norm"]}
    for l in range(cfg.NL):
        p, q = f"model.layers.{l}.", f"layers.{l}."
        sd[p + "self_attn.q_proj.weight"] = weights[q + "wq"]
        sd[p + "self_attn.k_proj.weight"] = weights[q + "wk"]
        sd[p + "self_attn.v_proj.weight"] = weights[q + "wv"]
        sd[p + "self_attn.o_proj.weight"] = weights[q + "wo"]
        sd[p + "mlp.gate_proj.weight"] = weights[q + "w_gate"]
        sd[p + "mlp.up_proj.weight"] = weights[q + "w_up"]
        sd[p + "mlp.down_proj.weight"] = weights[q + "w_down"]
        sd[p + "input_layernorm.weight"] = weights[q + "attn_norm"]
        sd[p + "post_attention_layernorm.weight"] = weights[q + "ffn_norm"]
    missing = m.load_state_dict({k: v.double() for k, v in sd.items()}, strict=False)
    assert not [k for k in missing.missing_keys if "rotary" not in k]
    return m


def test_sequential_decoder_equals_hf_llama():
    """The LLaMA-family base model (section 5): the oracle's one-token-at-a-time
    forward against the transformers library's implementation, same weights."""
    cfg = small_shape()
    W = make_weights(cfg, gain_std=0.2, std=0.3)
    m = oracle_model(cfg, W)
    hf = _hf_llama(cfg, W)
    prompt = uniform_tokens(7, 0, 11, cfg.V).tolist()
    with torch.no_grad():
        out = hf(torch.tensor([prompt]), output_hidden_states=True)
    cache = O.FlatCache(m, 32)
    for pos, t in enumerate(prompt):
        h, lg = O.ar_forward_token(m, cache, t, pos)
        np.testing.assert_allclose(lg, out.logits[0, pos].numpy(), rtol=0, atol=_HF_TOL)
        np.testing.assert_allclose(h, out.hidden_states[-1][0, pos].numpy(), rtol=0, atol=_HF_TOL)


def test_tree_verify_equals_hf_llama_with_4d_mask():
    """Section 2: pack the tree into one sequence and mask so that a token sees
    only its ancestors.  The library model is driven with exactly that: custom
    position ids and an explicit additive 4-D mask."""
    cfg = small_shape()
    W = make_weights(cfg, gain_std=0.2, std=0.3)
    m = oracle_model(cfg, W)
    hf = _hf_llama(cfg, W)
    tree = O.Tree(frozen_tree("tiny16"))
    L = 9
    prompt = uniform_tokens(8, 0, L, cfg.V).tolist()
    tok = uniform_tokens(8, 1, tree.T, cfg.V).tolist()
    cache = O.FlatCache(m, L + tree.T)
    O.ar_prefill(m, cache, prompt)
    hid, logits, _ = O.tree_verify(m, cache, L, tree, tok)
    # library side: one packed sequence prompt + tree tokens
    n = L + tree.T
    allow = torch.zeros(n, n, dtype=torch.bool)
    allow[:L, :L] = torch.tril(torch.ones(L, L, dtype=torch.bool))
    for a in range(tree.T):
        allow[L + a, :L] = True
        b = a
        while b >= 0:                       # walk up the parents (independent of the oracle's helper)
            allow[L + a, L + b] = True
            b = tree.parent[b]
    add = torch.zeros(n, n, dtype=torch.float64).masked_fill(~allow, float("-inf"))
    pos = torch.tensor([list(range(L)) + [L + tree.depth[a] for a in range(tree.T)]])
    with torch.no_grad():
        out = hf(torch.tensor([prompt + tok]), attention_mask=add[None, None], position_ids=pos,
                 output_hidden_states=True)
    np.testing.assert_allclose(logits, out.logits[0, L:].numpy(), rtol=0, atol=_HF_TOL)
    np.testing.assert_allclose(hid, out.hidden_states[-1][0, L:].numpy(), rtol=0, atol=_HF_TOL)


def test_chain_mask_is_causal_attention_sdpa():
    """A chain tree is ordinary causal attention (library: torch SDPA)."""
    rng = np.random.default_rng(3)
    T, L, Dh = 7, 5, 16
    q = rng.standard_normal((T, Dh)) * 2
    k = rng.standard_normal((L + T, Dh)) * 2
    v = rng.standard_normal((L + T, Dh))
    got = O.tree_attention(q, k, v, L, O.Tree(chain_tree(T)))
    mask = torch.ones(T, L + T, dtype=torch.bool).tril(diagonal=L)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.tensor(q)[None], torch.tensor(k)[None], torch.tensor(v)[None], attn_mask=mask[None])[0]
    np.testing.assert_allclose(got, ref.numpy(), atol=1e-12)


# ------------------------------------------------------------------ invariants of the paper
@pytest.mark.parametrize("tree_name", ["tiny16", "chain5", "star6", "random12"])
def test_I1_tree_verify_equals_sequential_on_every_path(tree_name):
    cfg = small_shape()
    W = make_weights(cfg, gain_std=0.2, std=0.3)
    m = oracle_model(cfg, W)
    parent = {"tiny16": frozen_tree("tiny16"), "chain5": chain_tree(5), "star6": star_tree(6),
              "random12": random_tree(12, 4, 5)}[tree_name]
    tree = O.Tree(parent)
    L = 6
    prompt = uniform_tokens(11, 0, L, cfg.V).tolist()
    tok = uniform_tokens(11, 1, tree.T, cfg.V).tolist()
    cache = O.FlatCache(m, L + tree.T)
    O.ar_prefill(m, cache, prompt)
    hid, logits, amax = O.tree_verify(m, cache, L, tree, tok)
    leaves = [n for n in range(tree.T) if not tree.children[n]]
    for leaf in leaves:
        path = tree.path(leaf)
        c2 = O.FlatCache(m, L + len(path))
        O.ar_prefill(m, c2, prompt)
        for j, n in enumerate(path):
            h, lg = O.ar_forward_token(m, c2, tok[n], L + j)
            np.testing.assert_allclose(lg, logits[n], atol=1e-10)
            np.testing.assert_allclose(h, hid[n], atol=1e-10)
            assert O.argmax_lowest(lg) == amax[n]
            # the node's K/V sit at scratch slot L + n and equal the sequential ones
            np.testing.assert_allclose(cache.K[:, L + n], c2.K[:, L + j], atol=1e-11)
            np.testing.assert_allclose(cache.V[:, L + n], c2.V[:, L + j], atol=1e-11)


def _scripted_hook(truth, tree, depth_of_step):
    """Plant the true greedy continuation along the rank-0 chain down to a
    scripted depth, keeping sibling tokens distinct (test harness, not method)."""
    def hook(tok, n_emitted):
        tok = list(tok)
        want = depth_of_step(n_emitted)
        cur = 0
        for j in range(1, want + 1):
            if not tree.children[cur] or n_emitted + j >= len(truth):
                break
            c = tree.children[cur][0]
            t = truth[n_emitted + j]
            for s in tree.children[cur]:
                if tok[s] == t:
                    tok[s] = tok[c]
            tok[c] = t
            cur = c
        return tok
    return hook


@pytest.mark.parametrize("tree_name,heads", [("tiny16", "random"), ("chain4", "random"), ("star6", "zero"),
                                              ("random12", "random"), ("single", "random"), ("tiny16", "scripted")])
def test_I2_hydra_greedy_equals_autoregressive_greedy(tree_name, heads):
    cfg = small_shape()
    W = make_weights(cfg, gain_std=0.2, std=0.3)
    if heads == "zero":
        W = {k: (torch.zeros_like(v) if k.startswith("heads.") else v) for k, v in W.items()}
    m = oracle_model(cfg, W)
    parent = {"tiny16": frozen_tree("tiny16"), "chain4": chain_tree(4), "star6": star_tree(6),
              "random12": random_tree(12, 3, 9), "single": [-1]}[tree_name]
    tree = O.Tree(parent)
    prompt = uniform_tokens(21, 0, 10, cfg.V).tolist()
    n_new = 14
    truth = O.ar_generate(m, prompt, n_new + 8)
    hook = None
    if heads == "scripted":
        depths = [3, 0, 2, 1, 3, 3, 1, 2, 0, 3, 2, 1, 3, 0, 1, 2, 3, 3]
        hook = _scripted_hook(truth, tree, lambda n: depths[n % len(depths)])
    out, acc = O.hydra_generate(m, tree, prompt, n_new, draft_hook=hook)
    assert out == truth[:n_new]
    assert all(1 <= a <= tree.max_depth + 1 for a in acc)
    assert sum(acc) >= n_new
    if heads == "scripted":
        assert max(acc) == tree.max_depth + 1 and min(acc) == 1     # both extremes exercised
    if tree_name == "single":
        assert all(a == 1 for a in acc)                              # T = 1 is plain decoding


def test_I3_cache_after_compaction_equals_autoregressive_cache():
    cfg = small_shape()
    W = make_weights(cfg, gain_std=0.2, std=0.3)
    m = oracle_model(cfg, W)
    tree = O.Tree(frozen_tree("tiny16"))
    prompt = uniform_tokens(31, 0, 9, cfg.V).tolist()
    truth = O.ar_generate(m, prompt, 24)
    depths = [2, 3, 1, 0, 3, 2]
    hook = _scripted_hook(truth, tree, lambda n: depths[n % len(depths)])
    cache = O.FlatCache(m, 80)
    L, h_last, root, _ = O.ar_prefill(m, cache, prompt)
    emitted = []
    for _ in range(5):
        n0 = len(emitted)
        e, L, h_last, root, info = O.hydra_step(m, cache, tree, L, h_last, root, lambda t: hook(t, n0))
        emitted += e
    assert emitted == truth[:len(emitted)] and root == truth[len(emitted)]
    ref = O.FlatCache(m, 80)
    h_ref = None
    for pos, t in enumerate(prompt + emitted):
        h_ref, _ = O.ar_forward_token(m, ref, t, pos)
    assert L == len(prompt) + len(emitted)
    np.testing.assert_allclose(cache.K[:, :L], ref.K[:, :L], atol=1e-11)
    np.testing.assert_allclose(cache.V[:, :L], ref.V[:, :L], atol=1e-11)
    np.testing.assert_allclose(h_last, h_ref, atol=1e-10)


def test_I5_medusa_special_case_path_independent():
    """Zero the embedding columns of every W1: the draft distribution at depth i
    no longer depends on the path, so all nodes of one depth get the same
    children (the independence equation of section 3)."""
    cfg = small_shape()
    W = make_weights(cfg, std=0.3)
    for i in range(1, cfg.K + 1):
        w1 = W[f"heads.{i}.w1"].clone()
        w1[:, cfg.d:] = 0
        W[f"heads.{i}.w1"] = w1
    m = oracle_model(cfg, W)
    tree = O.Tree(frozen_tree("tiny16"))
    h = np.random.default_rng(0).standard_normal(cfg.d)
    tok, _ = O.draft_tree(m, tree, h, root=5)
    tok2, _ = O.draft_tree(m, tree, h, root=77)
    assert tok[1:] == tok2[1:]
    for dpt in range(tree.max_depth):
        lists = [[tok[c] for c in tree.children[n]] for n in range(tree.T)
                 if tree.depth[n] == dpt and tree.children[n]]
        longest = max(lists, key=len)
        for l in lists:
            assert l == longest[:len(l)]


def test_I6_sequential_dependence_is_confined_to_the_subtree():
    cfg = small_shape()
    W = make_weights(cfg, std=0.3)
    m = oracle_model(cfg, W)
    tree = O.Tree(frozen_tree("tiny16"))
    h = np.random.default_rng(1).standard_normal(cfg.d)
    tok, _ = O.draft_tree(m, tree, h, root=5)
    forced = list(tok)
    forced[1] = (tok[1] + 1) % cfg.V                      # change one depth-1 candidate
    tok_b, logits_b = O.draft_tree(m, tree, h, root=5, forced_tokens=forced)
    _, logits_a = O.draft_tree(m, tree, h, root=5, forced_tokens=tok)
    in_subtree = lambda n: 1 in tree.path(n)
    changed = [n for n in logits_a if not np.allclose(logits_a[n], logits_b[n], atol=1e-14)]
    assert changed and all(in_subtree(n) for n in changed)
    assert all(n in changed for n in logits_a if in_subtree(n))
    # the root token matters to every head (x_t is an input of f_Hydra,i)
    _, logits_c = O.draft_tree(m, tree, h, root=6, forced_tokens=tok)
    assert all(not np.allclose(logits_a[n], logits_c[n], atol=1e-14) for n in logits_a)


# ------------------------------------------------------------------ closed forms / brute force
def test_head_closed_form_selector_weights():
    """Head i with selector weights: W1 picks chosen coordinates of
    u = [h ; E[x_t] ; E[x^_1] ...], Wout is a permutation, so the children are
    a sort of SiLU of known numbers.  Checks the concat order and which tokens
    of the path enter which slot."""
    d, V = 4, 6
    cfg = small_shape(d=d, H=2, Dh=2, F=8, V=V, K=2, NL=1)
    E = (np.arange(V * d, dtype=np.float64).reshape(V, d) - 10.0) / 8.0     # exact binary fractions
    W = make_weights(cfg)
    W["embed"] = torch.tensor(E)
    # head 1: u = [h(4); E[root](4)]; z = SiLU([h0, h3, E[root]_1, E[root]_2 + 0.5])
    w1 = np.zeros((d, 2 * d)); w1[0, 0] = 1; w1[1, 3] = 1; w1[2, 4 + 1] = 1; w1[3, 4 + 2] = 1
    W["heads.1.w1"] = torch.tensor(w1); W["heads.1.b1"] = torch.tensor([0.0, 0.0, 0.0, 0.5])
    wout = np.zeros((V, d)); wout[5, 0] = 1; wout[4, 1] = 1; wout[2, 2] = 1; wout[0, 3] = 1
    W["heads.1.wout"] = torch.tensor(wout)
    # head 2: u = [h; E[root]; E[tok(n)]]; z picks E[tok(n)]_0, E[root]_0, h1, h2
    w1 = np.zeros((d, 3 * d)); w1[0, 8 + 0] = 1; w1[1, 4 + 0] = 1; w1[2, 1] = 1; w1[3, 2] = 1
    W["heads.2.w1"] = torch.tensor(w1); W["heads.2.b1"] = torch.zeros(d)
    W["heads.2.wout"] = torch.tensor(np.eye(V, d))
    m = oracle_model(cfg, W)
    h = np.array([0.375, -2.0, 0.5, 1.0])
    root = 3                                               # E[3] = [0.25, 0.375, 0.5, 0.625]
    sil = lambda x: x / (1 + np.exp(-x))
    z1 = sil(np.array([0.375, 1.0, 0.375, 0.5 + 0.5]))
    lg1 = O.head_logits(m, 1, h, [root])
    np.testing.assert_allclose(lg1, [z1[3], 0, z1[2], 0, z1[1], z1[0]], atol=1e-15)
    # ids 0 and 4 tie at SiLU(1), ids 2 and 5 tie at SiLU(.375), ids 1 and 3 are 0
    assert O.top_k_ids(lg1, 4) == [0, 4, 2, 5]             # ties resolved by lowest id
    tree = O.Tree([-1, 0, 0, 1, 2])
    tok, _ = O.draft_tree(m, tree, h, root)
    assert tok[:3] == [3, 0, 4]
    # node 1 holds token 0 (E[0]_0 = -1.25) -> z = SiLU([-1.25, .25, -2, .5]) -> id 3
    # node 2 holds token 4 (E[4]_0 = +0.75) -> z = SiLU([ 0.75, .25, -2, .5]) -> id 0
    assert tok[3] == 3 and tok[4] == 0
    lg = O.head_logits(m, 2, h, [root, 4])
    np.testing.assert_allclose(lg[:4], sil(np.array([0.75, 0.25, -2.0, 0.5])), atol=1e-15)
    assert np.all(lg[4:] == 0)


def test_hydrapp_residual_layers_closed_form():
    """Section 3.1 "Scaling": extra MLP layers.  With W_j = 0, b_j = 0 a residual
    layer is the identity; with W_j = I it maps z to z + SiLU(z)."""
    cfg = small_shape(mlp_layers=3, K=1)
    W = make_weights(cfg, std=0.3)
    m0 = oracle_model(cfg.with_(mlp_layers=1), W)
    h = np.random.default_rng(2).standard_normal(cfg.d)
    base = O.head_logits(m0, 1, h, [4])
    for j in (2, 3):
        W[f"heads.1.w{j}"] = torch.zeros(cfg.d, cfg.d); W[f"heads.1.b{j}"] = torch.zeros(cfg.d)
    np.testing.assert_allclose(O.head_logits(oracle_model(cfg, W), 1, h, [4]), base, atol=1e-14)
    W["heads.1.w2"] = torch.eye(cfg.d)
    E = W["embed"].double().numpy()
    u = np.concatenate([h, E[4]])
    z = W["heads.1.w1"].double().numpy() @ u + W["heads.1.b1"].double().numpy()
    z = z / (1 + np.exp(-z))
    z = z + z / (1 + np.exp(-z))
    np.testing.assert_allclose(O.head_logits(oracle_model(cfg, W), 1, h, [4]),
                               W["heads.1.wout"].double().numpy() @ z, atol=1e-13)


def test_hydrapp_residual_layer_orientation_with_a_non_symmetric_matrix():
    """Section 3.1 "Scaling": layer j >= 2 is z + SiLU(W_j z + b_j) with W_j [out, in].  W_j holds two entries only,
    W_j[r, c] = 2 and W_j[c, q] = -1 (r, c, q distinct), so that W_j z is written out by hand element by element:
    (W z)[r] = 2 z[c], (W z)[c] = -z[q], zero elsewhere.  The transposed product would put 2 z[r] into element c and
    -z[c] into element q instead, which this comparison tells apart."""
    cfg = small_shape(mlp_layers=3, K=1)
    W = dict(make_weights(cfg, std=0.3))
    d = cfg.d
    h = np.random.default_rng(12).standard_normal(d)
    E = W["embed"].double().numpy()
    sil = lambda v: v / (1.0 + np.exp(-v))
    z = sil(W["heads.1.w1"].double().numpy() @ np.concatenate([h, E[4]]) + W["heads.1.b1"].double().numpy())   # layer 1: pinned by the selector tests
    for j, (r, c, q) in ((2, (3, 17, 5)), (3, (20, 1, 9))):
        Wj = torch.zeros(d, d); Wj[r, c] = 2.0; Wj[c, q] = -1.0
        W[f"heads.1.w{j}"] = Wj
        b = W[f"heads.1.b{j}"].double().numpy()
        pre = b.copy()
        pre[r] += 2.0 * z[c]
        pre[c] += -1.0 * z[q]
        z = z + sil(pre)
    want = W["heads.1.wout"].double().numpy() @ z
    got = O.head_logits(oracle_model(cfg, W), 1, h, [4])
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)
    # and the comparison does tell the transpose apart
    Wt = dict(W)
    for j in (2, 3):
        Wt[f"heads.1.w{j}"] = W[f"heads.1.w{j}"].t().contiguous()
    assert np.max(np.abs(O.head_logits(oracle_model(cfg, Wt), 1, h, [4]) - want)) > 1e-3


def test_P1_top_k_equals_full_stable_sort_with_planted_ties():
    rng = np.random.default_rng(5)
    for trial in range(50):
        V = int(rng.integers(3, 40))
        vals = rng.integers(-3, 4, size=V).astype(np.float64)      # many exact ties
        k = int(rng.integers(1, V + 1))
        ref = sorted(range(V), key=lambda i: (-vals[i], i))[:k]
        assert O.top_k_ids(vals, k) == ref
        assert O.argmax_lowest(vals) == ref[0]


def test_P2_accept_greedy_equals_brute_force_over_all_paths():
    rng = np.random.default_rng(6)
    for trial in range(200):
        T = int(rng.integers(1, 14))
        tree = O.Tree(random_tree(T, 4, 100 + trial))
        tok = rng.integers(0, 3, size=T).tolist()
        amax = rng.integers(0, 3, size=T).tolist()
        # make sibling tokens distinct, as a top-k always produces
        for n in range(T):
            seen = set()
            for c in tree.children[n]:
                while tok[c] in seen:
                    tok[c] += 3
                seen.add(tok[c])
        good = []
        for n in range(T):
            p = tree.path(n)
            if all(tok[p[j + 1]] == amax[p[j]] for j in range(len(p) - 1)):
                good.append(p)
        best = max(good, key=len)
        assert sum(len(p) == len(best) for p in good) == 1            # unique by distinct siblings
        n_acc, path, nxt, last = O.accept_greedy(tree, tok, amax)
        assert path == best and n_acc == len(best) and last == best[-1] and nxt == amax[best[-1]]
        assert 1 <= n_acc <= tree.max_depth + 1


def test_accept_duplicate_siblings_takes_lowest_node():
    tree = O.Tree([-1, 0, 0, 0])
    assert O.accept_greedy(tree, [9, 5, 5, 5], [5, 1, 2, 3])[1] == [0, 1]


def test_P3_closed_forms_rmsnorm_silu_softmax():
    rng = np.random.default_rng(7)
    x = rng.standard_normal((5, 64)) * 3
    y = O.rmsnorm(x, np.ones(64), 0.0)
    np.testing.assert_allclose(np.mean(y * y, axis=-1), 1.0, atol=1e-12)
    g = rng.standard_normal(64)
    np.testing.assert_allclose(O.rmsnorm(x, g, 0.0), y * g, atol=1e-12)
    np.testing.assert_allclose(O.rmsnorm(np.array([3.0, 4.0]), np.ones(2), 0.0), [3 / np.sqrt(12.5), 4 / np.sqrt(12.5)])
    # eps sits inside the square root, added to the mean square
    np.testing.assert_allclose(O.rmsnorm(np.array([1.0, 1.0]), np.ones(2), 3.0), [0.5, 0.5])
    assert O.silu(0.0) == 0.0
    np.testing.assert_allclose(O.silu(x) - O.silu(-x), x, atol=1e-12)
    np.testing.assert_allclose(O.silu(np.log(3.0)), np.log(3.0) * 0.75)
    p = O.softmax(x)
    np.testing.assert_allclose(p.sum(-1), 1.0, atol=1e-12)
    np.testing.assert_allclose(O.softmax(np.log(np.array([1.0, 2.0, 5.0]))), [0.125, 0.25, 0.625])
    np.testing.assert_allclose(O.softmax(x + 1000.0), p, atol=1e-12)


def test_P4_rope_properties():
    rng = np.random.default_rng(8)
    q, k = rng.standard_normal(16), rng.standard_normal(16)
    np.testing.assert_allclose(O.rope(q, 0, 10000.0), q)
    np.testing.assert_allclose(np.linalg.norm(O.rope(q, 37, 10000.0)), np.linalg.norm(q))
    d1 = O.rope(q, 12, 10000.0) @ O.rope(k, 5, 10000.0)
    d2 = O.rope(q, 107, 10000.0) @ O.rope(k, 100, 10000.0)
    np.testing.assert_allclose(d1, d2, atol=1e-12)
    # pairing j <-> j + Dh/2 and the rotation sense, on a unit vector: e_0 at
    # position 1 has frequency 1 -> (cos 1) e_0 + (sin 1) e_{Dh/2}
    e0 = np.zeros(8); e0[0] = 1
    want = np.zeros(8); want[0] = np.cos(1.0); want[4] = np.sin(1.0)
    np.testing.assert_allclose(O.rope(e0, 1, 10000.0), want, atol=1e-15)
    # slowest pair j = Dh/2 - 1 turns by theta^(-(Dh-2)/Dh) per position
    e3 = np.zeros(8); e3[3] = 1
    a = 3 * 10000.0 ** (-6.0 / 8.0)
    want = np.zeros(8); want[3] = np.cos(a); want[7] = np.sin(a)
    np.testing.assert_allclose(O.rope(e3, 3, 10000.0), want, atol=1e-15)


def test_P7_mask_one_hot_values_name_the_keys_seen():
    """Sharp scores + one-hot values: each output row is the indicator of the
    keys a node may see (prefix, ancestors and itself) times softmax weights."""
    tree = O.Tree(frozen_tree("tiny16"))
    T, L = tree.T, 3
    Dh = L + T
    q = np.zeros((T, Dh)); k = np.zeros((L + T, Dh))
    v = np.eye(L + T)
    out = O.tree_attention(q, k, v, L, tree)            # all scores equal -> uniform over allowed keys
    for n in range(T):
        allowed = set(range(L))
        a = n
        while a >= 0:
            allowed.add(L + a)
            a = tree.parent[a]
        row = np.zeros(L + T); row[list(allowed)] = 1.0 / len(allowed)
        np.testing.assert_allclose(out[n], row, atol=1e-15)


def test_kv_compact_moves_only_accepted_slots():
    cfg = small_shape()
    m = oracle_model(cfg, make_weights(cfg))
    cache = O.FlatCache(m, 20)
    rng = np.random.default_rng(9)
    cache.K[:] = rng.standard_normal(cache.K.shape); cache.V[:] = rng.standard_normal(cache.V.shape)
    K0, V0 = cache.K.copy(), cache.V.copy()
    L, path = 4, [0, 2, 7, 9]
    assert O.kv_compact(cache, L, path) == 8
    for j, n in enumerate(path):
        np.testing.assert_array_equal(cache.K[:, L + j], K0[:, L + n])
        np.testing.assert_array_equal(cache.V[:, L + j], V0[:, L + n])
    np.testing.assert_array_equal(cache.K[:, :L], K0[:, :L])
    np.testing.assert_array_equal(cache.K[:, L + 4:], K0[:, L + 4:])
