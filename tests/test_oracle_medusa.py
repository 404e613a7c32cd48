"""Pins for the oracle's Medusa-style draft heads (paper, section 2: "Lightweight heads as a draft model",
"Medusa decoding"; section 3, the displayed independence equation): p_draft = f_draft,i(h_{t-1}), one hidden
layer with a skip connection around it, no dependence on the candidate path.
"""
import numpy as np
import torch

from oracle import hydra_oracle as O
from synth import frozen_tree, uniform_tokens
from helpers import make_weights, oracle_model, small_shape


def test_children_do_not_depend_on_the_path():
    """Every node of depth i-1 gets a prefix of one and the same ranked list (section 3: no sequential dependence)."""
    cfg = small_shape(medusa=1)
    W = make_weights(cfg, std=0.3)
    m = oracle_model(cfg, W)
    tree = O.Tree(frozen_tree("tiny16"))
    h = np.random.default_rng(1).standard_normal(cfg.d)
    tok, lg = O.draft_tree(m, tree, h, 5)
    tok2, _ = O.draft_tree(m, tree, h, 77)                       # another root token: nothing but node 0 changes
    assert tok[1:] == tok2[1:]
    for i in range(1, tree.max_depth + 1):
        lists = [[tok[c] for c in tree.children[n]] for n in range(tree.T) if tree.depth[n] == i - 1 and tree.children[n]]
        longest = max(lists, key=len)
        assert all(l == longest[:len(l)] for l in lists)


def test_residual_form_closed_forms():
    """W1 = 0, b1 = 0: z = h, so the children are the top-k of Wout h.  W1 = 0, b1 = c: z = h + SiLU(c)."""
    cfg = small_shape(medusa=1, K=1)
    W = make_weights(cfg, std=0.3)
    W = dict(W)
    W["heads.1.w1"] = torch.zeros_like(W["heads.1.w1"]); W["heads.1.b1"] = torch.zeros_like(W["heads.1.b1"])
    m = oracle_model(cfg, W)
    h = np.random.default_rng(2).standard_normal(cfg.d)
    Wout = W["heads.1.wout"].double().numpy()
    np.testing.assert_allclose(O.head_logits(m, 1, h, [3]), Wout @ h, rtol=0, atol=1e-12)
    W["heads.1.b1"] = torch.full_like(W["heads.1.b1"], 0.75)
    m = oracle_model(cfg, W)
    s = 0.75 / (1.0 + np.exp(-0.75))
    np.testing.assert_allclose(O.head_logits(m, 1, h, [3]), Wout @ (h + s), rtol=0, atol=1e-12)


def test_first_layer_orientation_with_a_non_symmetric_matrix():
    """z = h + SiLU(W1 h + b1) with W1 [out, in] (section 2, "Medusa decoding": one hidden layer with a skip
    connection).  W1 holds W1[r, c] = 1.5 and W1[c, q] = -2 only, so W1 h is written out by hand:
    (W1 h)[r] = 1.5 h[c], (W1 h)[c] = -2 h[q]; the transposed product differs and is told apart."""
    cfg = small_shape(medusa=1, K=1)
    W = dict(make_weights(cfg, std=0.3))
    d = cfg.d
    r, c, q = 2, 11, 7
    W1 = torch.zeros(d, d); W1[r, c] = 1.5; W1[c, q] = -2.0
    W["heads.1.w1"] = W1
    h = np.random.default_rng(3).standard_normal(d)
    pre = W["heads.1.b1"].double().numpy().copy()
    pre[r] += 1.5 * h[c]
    pre[c] += -2.0 * h[q]
    z = h + pre / (1.0 + np.exp(-pre))
    want = W["heads.1.wout"].double().numpy() @ z
    np.testing.assert_allclose(O.head_logits(oracle_model(cfg, W), 1, h, [3]), want, rtol=0, atol=1e-12)
    Wt = dict(W); Wt["heads.1.w1"] = W1.t().contiguous()
    assert np.max(np.abs(O.head_logits(oracle_model(cfg, Wt), 1, h, [3]) - want)) > 1e-3


def test_greedy_output_unchanged_with_medusa_heads():
    cfg = small_shape(medusa=1)
    W = make_weights(cfg, gain_std=0.2, std=0.3)
    m = oracle_model(cfg, W)
    tree = O.Tree(frozen_tree("tiny16"))
    prompt = uniform_tokens(21, 0, 10, cfg.V).tolist()
    truth = O.ar_generate(m, prompt, 12)
    out, acc = O.hydra_generate(m, tree, prompt, 12)
    assert out == truth and all(1 <= a <= tree.max_depth + 1 for a in acc)
