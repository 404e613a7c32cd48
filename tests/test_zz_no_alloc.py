"""accept_typical_static (the entry point that allocates nothing: its scratch is a fixed device array inside the
library) against accept_typical, through the C ABI: integer outputs bit for bit, on two calls in a row, the second
with a smaller input, and the size limit is an error, not an access."""
import numpy as np
import pytest
import torch

from oracle import hydra_oracle as O
from synth import frozen_tree
from helpers import make_weights, small_shape
from gpu_util import gpu_session

pytestmark = pytest.mark.gpu


def _inputs(tree, B, V, seed):
    rng = np.random.default_rng(seed)
    T = tree.T
    logits = rng.standard_normal((B, T, V)).astype(np.float32) * 2.0
    tok = rng.integers(0, V, size=(B, T))
    for b in range(B):
        for c in range(1, T):
            if rng.random() < 0.75:
                logits[b, tree.parent[c], tok[b, c]] += float(rng.uniform(4.0, 14.0))
    return torch.tensor(tok, dtype=torch.int32, device="cuda:0"), torch.tensor(logits, device="cuda:0"), torch.tensor(rng.random(B).astype(np.float32), device="cuda:0")


def test_static_entry_point_equals_accept_typical_on_two_calls_in_a_row():
    parent = frozen_tree("prior64")
    tree = O.Tree(parent)
    V, Bmax = 1000, 5
    cfg = small_shape(d=128, NL=1, H=2, Dh=64, F=176, V=V, K=4, T=len(parent))
    sess = gpu_session(cfg, parent, Bmax, 32, make_weights(cfg), want_logits=True)
    P = tree.max_depth + 1
    lengths = set()
    for call, (B, use_u) in enumerate(((5, True), (2, False))):          # the second call is smaller
        tok, logits, u = _inputs(tree, B, V, 30 + call)
        outs = []
        for static in (False, True):
            n_acc = torch.full((B,), -7, dtype=torch.int32, device="cuda:0"); path = torch.full((B, P), -7, dtype=torch.int32, device="cuda:0")
            nxt = torch.full((B,), -7, dtype=torch.int32, device="cuda:0"); last = torch.full((B,), -7, dtype=torch.int32, device="cuda:0")
            if static:
                sess.main.accept_typical_static(B, tok, logits, 0.7, 0.15, float(np.sqrt(0.15)), u if use_u else None, n_acc, path, nxt, last)
            else:
                sess.main.accept_typical(B, sess.ws, tok, logits, 0.7, 0.15, float(np.sqrt(0.15)), u if use_u else None, n_acc, path, nxt, last)
            torch.cuda.synchronize()
            assert sess.main.read_flags() == 0
            outs.append((n_acc, path, nxt, last))
        for a, b in zip(*outs):
            assert torch.equal(a, b)
        assert int(outs[1][0].min()) >= 1
        lengths |= set(outs[1][0].tolist())
    assert len(lengths) >= 2                                              # paths of several lengths were exercised


def test_static_entry_point_rejects_more_nodes_than_its_buffer_holds():
    from paper_2402_05109_amd import binding as hb
    parent = frozen_tree("prior128")
    V = 64
    cfg = small_shape(d=128, NL=1, H=2, Dh=64, F=176, V=V, K=4, T=len(parent))
    B = 16384 // len(parent) + 1                                          # one row too many
    sess = gpu_session(cfg, parent, B, 16, make_weights(cfg), want_logits=True)
    o = sess.out()
    before = o.n_acc.clone()
    with pytest.raises(hb.HydraError) as e:
        sess.main.accept_typical_static(B, o.tree_tokens, o.logits, 0.7, 0.1, 0.3, None, o.n_acc, o.path, o.next_root, o.last_node)
    assert e.value.code == hb.E_CAPACITY and "16384" in str(e.value)
    torch.cuda.synchronize()
    assert torch.equal(o.n_acc, before)
    sess.main.accept_typical_static(B - 1, o.tree_tokens, o.logits, 0.7, 0.1, 0.3, None, o.n_acc, o.path, o.next_root, o.last_node)   # exactly at the limit
    torch.cuda.synchronize()
    assert sess.main.read_flags() == 0
