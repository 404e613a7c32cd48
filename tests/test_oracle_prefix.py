"""Pins for the oracle's Hydra++ prefix-attention layer (paper, section 3.1 item 3 and the appendix
paragraph "Hydra-specific prefix attention"): one extra decoder layer over the verified sequence whose
output at the last verified token is what the draft heads read.

None of these re-types the oracle's formulas: a library decoder layer, the two independent code paths of
the oracle against each other, closed forms, and the paper's invariant that greedy acceptance leaves the
generated text unchanged whatever the heads read.
"""
import numpy as np
import pytest
import torch

from oracle import hydra_oracle as O
from synth import frozen_tree, uniform_tokens
from helpers import make_weights, oracle_model, small_shape

_HF_TOL = 5e-6      # the library computes RMSNorm and rotary tables in fp32 (see test_oracle_pins.py)


def _setup(**kw):
    cfg = small_shape(prefix=1, **kw)
    W = make_weights(cfg, gain_std=0.2, std=0.3)
    return cfg, W, oracle_model(cfg, W)


def test_prefix_layer_equals_hf_llama_decoder_layer_on_given_hidden_states():
    """A one-layer transformers LLaMA fed `inputs_embeds`, with its final norm made the identity, is exactly
    'one pre-norm decoder layer applied to given hidden states'."""
    from transformers import LlamaConfig, LlamaModel
    cfg, W, m = _setup()
    hc = LlamaConfig(vocab_size=cfg.V, hidden_size=cfg.d, intermediate_size=cfg.F, num_hidden_layers=1,
                     num_attention_heads=cfg.H, num_key_value_heads=cfg.H, rms_norm_eps=cfg.rms_eps,
                     rope_theta=cfg.rope_theta, max_position_embeddings=256, attention_bias=False, mlp_bias=False,
                     hidden_act="silu", attn_implementation="eager")
    hf = LlamaModel(hc).double().eval()
    p = "layers.0."
    sd = {p + "self_attn.q_proj.weight": W["prefix.wq"], p + "self_attn.k_proj.weight": W["prefix.wk"],
          p + "self_attn.v_proj.weight": W["prefix.wv"], p + "self_attn.o_proj.weight": W["prefix.wo"],
          p + "mlp.gate_proj.weight": W["prefix.w_gate"], p + "mlp.up_proj.weight": W["prefix.w_up"],
          p + "mlp.down_proj.weight": W["prefix.w_down"], p + "input_layernorm.weight": W["prefix.attn_norm"],
          p + "post_attention_layernorm.weight": W["prefix.ffn_norm"]}
    missing = hf.load_state_dict({k: v.double() for k, v in sd.items()}, strict=False)
    assert sorted(k for k in missing.missing_keys if "rotary" not in k) == ["embed_tokens.weight", "norm.weight"]
    hf.norm = torch.nn.Identity()
    rng = np.random.default_rng(3)
    X = rng.standard_normal((9, cfg.d))
    with torch.no_grad():
        ref = hf(inputs_embeds=torch.tensor(X)[None]).last_hidden_state[0].numpy()
    pc = O.PrefixCache(m, 16)
    for pos in range(9):
        np.testing.assert_allclose(O.prefix_token(m, pc, X[pos], pos), ref[pos], rtol=0, atol=_HF_TOL)


@pytest.mark.parametrize("L,n", [(0, 1), (0, 7), (5, 1), (5, 4), (13, 5)])
def test_chunked_pass_equals_one_position_at_a_time(L, n):
    cfg, W, m = _setup()
    rng = np.random.default_rng(10 * L + n)
    X = rng.standard_normal((L + n, cfg.d))
    a, b = O.PrefixCache(m, 32), O.PrefixCache(m, 32)
    seq = np.stack([O.prefix_token(m, a, X[p], p) for p in range(L + n)])
    for p in range(L):
        O.prefix_token(m, b, X[p], p)
    out = O.prefix_chunk(m, b, L, X[L:])
    np.testing.assert_allclose(out, seq[L:], rtol=0, atol=1e-12)
    np.testing.assert_allclose(b.K[:L + n], a.K[:L + n], rtol=0, atol=1e-13)
    np.testing.assert_allclose(b.V[:L + n], a.V[:L + n], rtol=0, atol=1e-13)


def test_closed_forms_residual_only_and_first_position():
    cfg, W, m = _setup()
    rng = np.random.default_rng(4)
    x = rng.standard_normal(cfg.d)
    # both branches switched off: the layer is the identity
    W0 = dict(W); W0["prefix.wo"] = torch.zeros_like(W["prefix.wo"]); W0["prefix.w_down"] = torch.zeros_like(W["prefix.w_down"])
    m0 = oracle_model(cfg, W0)
    np.testing.assert_array_equal(O.prefix_token(m0, O.PrefixCache(m0, 4), x, 0), x)
    # position 0 attends to itself only: attention output = V row, whatever q and k are; with the FFN off
    # the layer is x + Wo Wv rmsnorm(x)
    W1 = dict(W); W1["prefix.w_down"] = torch.zeros_like(W["prefix.w_down"])
    m1 = oracle_model(cfg, W1)
    n1 = x / np.sqrt(np.mean(x * x) + cfg.rms_eps) * W["prefix.attn_norm"].double().numpy()
    want = x + W["prefix.wo"].double().numpy() @ (W["prefix.wv"].double().numpy() @ n1)
    np.testing.assert_allclose(O.prefix_token(m1, O.PrefixCache(m1, 4), x, 0), want, rtol=0, atol=1e-12)


def test_greedy_output_is_unchanged_and_heads_read_the_prefix_state():
    """Greedy acceptance returns the base model's greedy text whatever the draft heads read (section 5), so
    Hydra++ generation equals plain greedy decoding; with an identity prefix layer the drafts (hence the
    acceptance lengths) equal plain Hydra's, and with a real one they differ."""
    cfg, W, m = _setup()
    tree = O.Tree(frozen_tree("tiny16"))
    prompt = uniform_tokens(21, 0, 10, cfg.V).tolist()
    truth = O.ar_generate(m, prompt, 12)
    out_p, acc_p = O.hydra_generate(m, tree, prompt, 12, prefix=True)
    out_h, acc_h = O.hydra_generate(m, tree, prompt, 12, prefix=False)
    assert out_p == truth and out_h == truth
    W0 = dict(W); W0["prefix.wo"] = torch.zeros_like(W["prefix.wo"]); W0["prefix.w_down"] = torch.zeros_like(W["prefix.w_down"])
    m0 = oracle_model(cfg, W0)
    out_0, acc_0 = O.hydra_generate(m0, tree, prompt, 12, prefix=True)
    assert out_0 == truth and acc_0 == acc_h
    # first draft tree: identity layer -> same tokens as plain Hydra; real layer -> the head input differs
    cache, pc = O.FlatCache(m, 64), O.PrefixCache(m, 64)
    g = None
    for pos, t in enumerate(prompt):
        h, lg = O.ar_forward_token(m, cache, t, pos)
        g = O.prefix_token(m, pc, h, pos)
    root = O.argmax_lowest(lg)
    tok_plain, _ = O.draft_tree(m, tree, h, root)
    tok_prefix, _ = O.draft_tree(m, tree, g, root)
    assert np.max(np.abs(g - h)) > 1e-3
    assert list(tok_plain) != list(tok_prefix)


def test_step_feeds_the_accepted_tokens_in_order():
    """After a step that accepts several tokens the prefix cache must equal the one obtained by feeding the
    base hidden states of the same tokens one by one (the layer sees the verified sequence, nothing else)."""
    cfg, W, m = _setup()
    tree = O.Tree(frozen_tree("tiny16"))
    prompt = uniform_tokens(5, 0, 9, cfg.V).tolist()
    truth = O.ar_generate(m, prompt, 8)
    # scripted drafts: the left-most path carries the true continuation, so 4 tokens are accepted
    def hook(tok):
        tok = list(tok); cur = 0
        for j in range(tree.max_depth):
            c = tree.children[cur][0]; tok[c] = truth[1 + j]; cur = c
        return tok
    cache, pc = O.FlatCache(m, 64), O.PrefixCache(m, 64)
    for pos, t in enumerate(prompt):
        h, lg = O.ar_forward_token(m, cache, t, pos)
        g = O.prefix_token(m, pc, h, pos)
    emitted, L2, h_new, root2, info = O.hydra_step(m, cache, tree, len(prompt), g, O.argmax_lowest(lg), hook, pc)
    assert info["n_acc"] == tree.max_depth + 1 and emitted == truth[:tree.max_depth + 1]
    # reference: plain sequential base + prefix over prompt + emitted tokens
    c2, p2 = O.FlatCache(m, 64), O.PrefixCache(m, 64)
    for pos, t in enumerate(prompt + emitted):
        h, _ = O.ar_forward_token(m, c2, t, pos)
        g2 = O.prefix_token(m, p2, h, pos)
    np.testing.assert_allclose(pc.K[:L2], p2.K[:L2], rtol=0, atol=1e-9)
    np.testing.assert_allclose(pc.V[:L2], p2.V[:L2], rtol=0, atol=1e-9)
    np.testing.assert_allclose(h_new, g2, rtol=0, atol=1e-9)
