"""Faults that must surface as device flags, never as a wrong silent result or an access out of bounds: values too
large for the 16-bit interior of the bf16 family, weights too small for it, page-table entries outside the cache,
paths that are not strictly increasing, rows over capacity in kv_compact.  Every kernel exits normally in every case."""
import numpy as np
import pytest
import torch

from synth import frozen_tree, uniform_tokens
from helpers import make_weights
from gpu_util import gpu_session
from test_gpu_bf16 import bf16_shape

pytestmark = pytest.mark.gpu
SATURATED, WEIGHT_UNDERFLOW, BAD_PAGE, BAD_PATH, CAPACITY = 16, 32, 64, 4, 1


def _verify(sess, T, V, L):
    o = sess.out()
    o.tree_tokens.copy_(uniform_tokens(5, 0, sess.B * T, V).reshape(sess.B, T).to(torch.int32))
    sess.seq_len.fill_(L); sess.host_len = L
    sess.verify()
    torch.cuda.synchronize()
    return o


@pytest.mark.parametrize("layer_kernel", ["0", "1"])
def test_values_beyond_half_range_raise_the_saturation_flag(layer_kernel, monkeypatch):
    monkeypatch.setenv("HYDRA_LAYER_KERNEL", layer_kernel)
    cfg = bf16_shape()
    W = dict(make_weights(cfg, gain_std=0.1, std=0.05))
    parent = frozen_tree("tiny16")
    sess = gpu_session(cfg, parent, 1, 64, W, want_logits=True)
    o = _verify(sess, len(parent), cfg.V, 20)
    assert sess.main.read_flags() == 0                                    # ordinary weights: nothing clamps
    # a norm gain of 1e7 puts x * gain (the GEMM input before the division by the rms) far beyond 65504
    W["layers.1.attn_norm"] = torch.full_like(W["layers.1.attn_norm"], 1.0e7)
    sess = gpu_session(cfg, parent, 1, 64, W, want_logits=True)
    o = _verify(sess, len(parent), cfg.V, 20)
    assert sess.main.read_flags() & SATURATED
    assert bool(torch.isfinite(o.hidden).all()) and bool(torch.isfinite(o.logits).all())      # clamped, not NaN


def test_a_weight_too_small_for_the_interior_is_flagged_at_load_time():
    cfg = bf16_shape()
    W = dict(make_weights(cfg))
    parent = frozen_tree("tiny16")
    sess = gpu_session(cfg, parent, 1, 32, W)
    assert sess.main.read_flags() == 0
    w = W["layers.0.wo"].clone()
    w[3, 5] = 2.0 ** -26                                                  # a bfloat16 value; zero as a half
    W["layers.0.wo"] = w
    sess = gpu_session(cfg, parent, 1, 32, W)
    assert sess.main.read_flags() == WEIGHT_UNDERFLOW


@pytest.mark.parametrize("dtype,layer_kernel", [("bf16", "0"), ("bf16", "1"), ("f32", "0")])
def test_a_page_id_outside_the_cache_is_flagged_not_followed(dtype, layer_kernel, monkeypatch):
    monkeypatch.setenv("HYDRA_LAYER_KERNEL", layer_kernel)
    cfg = bf16_shape(dtype=dtype)
    W = make_weights(cfg, std=0.05)
    parent = frozen_tree("tiny16")
    T, L = len(parent), 40
    sess = gpu_session(cfg, parent, 2, 96, W, want_logits=True)
    o = _verify(sess, T, cfg.V, L)
    assert sess.main.read_flags() == 0
    pt = sess.page_table.clone()
    for bad_entry, bad_value in ((1, 10 ** 6), (L // 16, -3)):             # a page of the prefix, then the page the tree slots start in
        sess.page_table.copy_(pt)
        sess.page_table[1, bad_entry] = bad_value
        o = _verify(sess, T, cfg.V, L)
        assert sess.main.read_flags() & BAD_PAGE
        # the same through accept + compact: the copies of row 1 touch the bad page only if its path moves a slot there
        o.n_acc.fill_(2); o.path.fill_(-1); o.path[:, 0] = 0; o.path[:, 1] = 3; o.last_node.fill_(3); o.next_root.fill_(1)
        sess.seq_len.fill_(L)
        sess.compact()
        torch.cuda.synchronize()
        fl = sess.main.read_flags()
        assert fl in (0, BAD_PAGE)
    sess.page_table.copy_(pt)


def test_kv_compact_rejects_a_path_that_is_not_strictly_increasing_and_leaves_overflowing_rows_alone():
    cfg = bf16_shape()
    W = make_weights(cfg, std=0.05)
    parent = frozen_tree("tiny16")
    T, L = len(parent), 20
    sess = gpu_session(cfg, parent, 2, 64, W, want_logits=True)
    o = _verify(sess, T, cfg.V, L)
    assert sess.main.read_flags() == 0
    o.n_acc.fill_(3); o.path.fill_(-1)
    o.path[0, :3] = torch.tensor([0, 5, 2], dtype=torch.int32)            # goes back: not a root path
    o.path[1, :3] = torch.tensor([0, 1, 5], dtype=torch.int32)
    o.last_node.copy_(torch.tensor([2, 5], dtype=torch.int32)); o.next_root.fill_(7)
    sess.compact()
    torch.cuda.synchronize()
    assert sess.main.read_flags() == BAD_PATH
    # a row over capacity: verify flags it and skips it; compact then keeps its state
    sess.seq_len.copy_(torch.tensor([L, sess.kv.max_pages * 16 - 3], dtype=torch.int32))
    sess.host_len = L
    sess.h_last.fill_(0.25); sess.root.fill_(11)
    o.tree_tokens.copy_(uniform_tokens(5, 1, 2 * T, cfg.V).reshape(2, T).to(torch.int32))
    sess.verify(); sess.accept(); sess.compact()
    torch.cuda.synchronize()
    assert sess.main.read_flags() & CAPACITY
    assert int(sess.seq_len[1]) == sess.kv.max_pages * 16 - 3 and int(sess.root[1]) == 11
    assert bool((sess.h_last[1] == 0.25).all()) and bool((o.kv_index[1] == -1).all())
    assert int(sess.seq_len[0]) == L + int(o.n_acc[0]) and int(sess.root[0]) == int(o.next_root[0])
