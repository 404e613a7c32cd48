"""The hot path under HIP graph capture, and run-to-run determinism.

The calls allocate nothing, never synchronise and record no memset, so a whole step can be captured into a graph
by the caller.  The check follows the usual protocol for graphs on this hardware: the graph is replayed several
times with eager work and synchronisations in between, and every replay is compared with the eager result of the
same state, bit for bit (all reductions in the kernels have a fixed order, so equal inputs give equal bits).
"""
import pytest
import torch

from synth import frozen_tree, uniform_tokens
from helpers import make_weights, small_shape
from gpu_util import gpu_session

pytestmark = pytest.mark.gpu


def _outputs(sess):
    o = sess.out()
    return [t.clone() for t in (o.tree_tokens, o.argmax, o.hidden, o.n_acc, o.path, o.next_root, sess.h_last, sess.root, sess.seq_len)]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_step_replays_from_a_graph_bit_exactly(dtype):
    if dtype == "bf16":
        cfg = small_shape(dtype="bf16", d=256, NL=2, H=2, Dh=128, F=384, V=1000, K=3, T=16, prefix=1)
    else:
        cfg = small_shape(d=128, NL=2, H=2, Dh=64, F=176, V=300, K=3, T=16)
    W = make_weights(cfg)
    B = 2
    sess = gpu_session(cfg, frozen_tree("tiny16"), B, 96, W, prefill_chunk=8)
    sess.prefill(torch.stack([uniform_tokens(3, b, 20, cfg.V) for b in range(B)]))
    sess.sync_len()
    sess.host_len += 32                         # the hint is frozen into the graph: an upper bound for all replays below
    hint = sess.host_len

    def state():
        s = [sess.seq_len.clone(), sess.h_last.clone(), sess.root.clone()]
        if sess.prefix:
            s.append(sess.pseq_len.clone())
        return s

    def restore(s):
        sess.seq_len.copy_(s[0]); sess.h_last.copy_(s[1]); sess.root.copy_(s[2])
        if sess.prefix:
            sess.pseq_len.copy_(s[3])
        sess.host_len = hint

    def eager_step():
        sess.host_len = hint
        sess.step()

    # determinism first: the same state twice
    s0 = state()
    eager_step(); torch.cuda.synchronize(); a = _outputs(sess)
    restore(s0)
    eager_step(); torch.cuda.synchronize(); b = _outputs(sess)
    assert all(torch.equal(x, y) for x, y in zip(a, b)), "two eager runs of the same state differ"

    # capture (torch captures on a side stream; the binding passes the current stream to every call)
    restore(s0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        eager_step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    restore(s0)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        sess.host_len = hint
        sess.step()
    torch.cuda.synchronize()

    # replays from successive states, each checked against the eager result of the same state
    cur = s0
    for it in range(4):
        restore(cur)
        eager_step(); torch.cuda.synchronize()
        want, nxt = _outputs(sess), state()
        scratch = torch.randn(1 << 16, device="cuda:0").sum().item()        # unrelated eager work and a synchronisation in between
        restore(cur)
        g.replay(); torch.cuda.synchronize()
        got = _outputs(sess)
        assert all(torch.equal(x, y) for x, y in zip(want, got)), f"replay {it} differs from the eager step"
        cur = nxt
    assert sess.main.read_flags() == 0
