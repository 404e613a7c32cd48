"""The persistent layer kernel (all decoder layers of a tree_verify_forward of up to 64 rows as one kernel with
grid-wide hand-offs, csrc/bf16_layers.hip), switched on through its environment variable: parity against the float64
oracle with the tolerances of the 16-bit family, bit-identical repeats, agreement with the multi-kernel path, and the
give-up path of its bounded waits (forced from the host: every workgroup still exits normally)."""
import numpy as np
import pytest
import torch

from synth import frozen_tree, uniform_tokens
from helpers import make_weights
from gpu_util import gpu_session
from test_gpu_bf16 import TREES, _verify_forward_teacher_forced, bf16_shape

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("tree_name,B,L", [("prior64", 1, 37), ("tiny16", 3, 17), ("single", 2, 90), ("chain40", 1, 0),
                                            ("prior32", 2, 200), ("tiny16", 4, 1000), ("prior64", 1, 500)])
def test_layer_kernel_matches_oracle(tree_name, B, L, monkeypatch):
    monkeypatch.setenv("HYDRA_LAYER_KERNEL", "1")
    _verify_forward_teacher_forced(tree_name, B, L)


def _run(sess, toks, lens):
    o = sess.out()
    sess.seq_len.copy_(torch.tensor(lens, dtype=torch.int32)); sess.host_len = max(lens)
    o.tree_tokens.copy_(toks)
    sess.verify()
    torch.cuda.synchronize()
    return o.hidden.clone(), o.logits.clone(), o.argmax.clone(), o.margin.clone()


def _setup(B, lens, tree="tiny16"):
    cfg = bf16_shape()
    W = make_weights(cfg, gain_std=0.1, std=0.05)
    parent = TREES[tree]()
    T = len(parent)
    sess = gpu_session(cfg, parent, B, max(lens) + 64, W, page_perm_seed=3, want_logits=True)
    rng = np.random.default_rng(8)
    for l in range(cfg.NL):
        t = torch.tensor(rng.standard_normal((B, max(lens), 2, cfg.H, cfg.Dh)) * 0.5, dtype=torch.float32, device="cuda:0")
        sess.main.kv_write(B, l, sess.kv, 0, max(lens), t)
    toks = torch.stack([uniform_tokens(8, b, T, cfg.V) for b in range(B)]).to(torch.int32)
    return cfg, sess, toks


def test_layer_kernel_is_used_repeatable_and_close_to_the_multi_kernel_path(monkeypatch):
    lens = [150, 1, 37]
    cfg, sess, toks = _setup(3, lens)
    assert sess.main.layer_kernel_info(3)[0] == 1
    monkeypatch.setenv("HYDRA_LAYER_KERNEL", "0")
    ref = _run(sess, toks, lens)
    assert sess.main.read_flags() == 0
    monkeypatch.setenv("HYDRA_LAYER_KERNEL", "1")
    a = _run(sess, toks, lens)
    b = _run(sess, toks, lens)
    assert sess.main.read_flags() == 0
    for x, y in zip(a, b):
        assert torch.equal(x, y)                          # every sum has a fixed order
    scale = float(ref[1].abs().max())
    assert float((a[1] - ref[1]).abs().max()) <= 5e-3 * scale and not torch.equal(a[1], ref[1])   # other split of K: rounding only, and really the other path
    assert float((a[0] - ref[0]).abs().max()) <= 5e-3 * float(ref[0].abs().max())


def test_layer_kernel_gives_up_with_a_flag_when_a_hand_off_cannot_complete(monkeypatch):
    """One group more than exists is awaited and the spin limit is tiny: no hand-off can complete, every workgroup leaves
    through its bounded wait, the call returns, bit 3 of the flags is set; the next ordinary call is correct again."""
    lens = [40]
    cfg, sess, toks = _setup(1, lens)
    monkeypatch.setenv("HYDRA_LAYER_KERNEL", "1")
    good = _run(sess, toks, lens)
    assert sess.main.read_flags() == 0
    monkeypatch.setenv("HYDRA_LAYER_KERNEL_TEST_STALL", "1")
    monkeypatch.setenv("HYDRA_LAYER_KERNEL_SPIN", "200")
    _run(sess, toks, lens)
    assert sess.main.read_flags() & 8
    monkeypatch.delenv("HYDRA_LAYER_KERNEL_TEST_STALL")
    monkeypatch.delenv("HYDRA_LAYER_KERNEL_SPIN")
    again = _run(sess, toks, lens)
    assert sess.main.read_flags() == 0
    for x, y in zip(good, again):
        assert torch.equal(x, y)


def test_long_or_unknown_contexts_take_the_multi_kernel_path(monkeypatch):
    """Without an upper bound of the row lengths (seq_len_hint = 0) the layer kernel is not used: results equal the
    multi-kernel path bit for bit."""
    lens = [33]
    cfg, sess, toks = _setup(1, lens)
    monkeypatch.setenv("HYDRA_LAYER_KERNEL", "0")
    ref = _run(sess, toks, lens)
    monkeypatch.setenv("HYDRA_LAYER_KERNEL", "1")
    o = sess.out()
    sess.seq_len.copy_(torch.tensor(lens, dtype=torch.int32))
    o.tree_tokens.copy_(toks)
    sess.kv.seq_len_hint = 0
    sess.main.tree_verify_forward(1, sess.ws, o.tree_tokens, sess.seq_len, sess.kv, o.hidden, o.argmax, o.margin, o.logits)
    torch.cuda.synchronize()
    assert torch.equal(o.logits, ref[1]) and torch.equal(o.hidden, ref[0])
