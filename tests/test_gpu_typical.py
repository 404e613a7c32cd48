"""GPU parity of accept_typical (typical acceptance: paper, section 6.3) against the oracle, through the C ABI.

The call works on logits, so the inputs are seeded synthetic logits with planted high-probability candidates
(shapes of the workloads: V = 32000 / ragged 1000, the frozen 64- and 16-node trees, several rows).  All
outputs are integers and must be bit-exact, except where float32 decides them inside rounding: a row is
excluded, and counted, if some candidate's probability is within 1e-4 (relative) of its threshold, and the
sampled token is not compared if u lies within 1e-5 of a step of the cumulative distribution.
"""
import numpy as np
import pytest
import torch

from oracle import hydra_oracle as O
from synth import frozen_tree, random_tree
from helpers import make_weights, small_shape
from gpu_util import gpu_session

pytestmark = pytest.mark.gpu


def _session(parent, B, V):
    cfg = small_shape(d=128, NL=1, H=2, Dh=64, F=176, V=V, K=4, T=len(parent))
    return gpu_session(cfg, parent, B, 32, make_weights(cfg), want_logits=True), cfg


@pytest.mark.parametrize("tree_name,V,B,use_u", [("prior64", 32000, 3, True), ("tiny16", 1000, 5, True), ("prior64", 1000, 2, False),
                                                 ("single", 257, 2, True), ("random40", 4099, 4, True)])
def test_accept_typical_matches_oracle(tree_name, V, B, use_u):
    parent = {"prior64": frozen_tree("prior64"), "tiny16": frozen_tree("tiny16"), "single": [-1],
              "random40": random_tree(40, 4, 11)}[tree_name]
    tree = O.Tree(parent)
    T = tree.T
    sess, cfg = _session(parent, B, V)
    rng = np.random.default_rng(V + T)
    tau, eps = 0.7, 0.15
    alpha = float(np.sqrt(eps))
    logits = rng.standard_normal((B, T, V)).astype(np.float32) * 2.0
    tok = rng.integers(0, V, size=(B, T))
    for b in range(B):                               # plant candidates of graded probability so that paths of all lengths occur
        for c in range(1, T):
            r = rng.random()
            if r < 0.75:
                logits[b, tree.parent[c], tok[b, c]] += float(rng.uniform(4.0, 14.0))
    u = rng.random(B).astype(np.float32) if use_u else None
    o = sess.out()
    o.tree_tokens.copy_(torch.tensor(tok, dtype=torch.int32))
    o.logits.copy_(torch.tensor(logits))
    ud = torch.tensor(u, device="cuda:0") if use_u else None
    sess.main.accept_typical(B, sess.ws, o.tree_tokens, o.logits, tau, eps, alpha, ud, o.n_acc, o.path, o.next_root, o.last_node)
    torch.cuda.synchronize()
    assert sess.main.read_flags() == 0
    compared = skipped = sampled = 0
    lengths = set()
    for b in range(B):
        lg = logits[b].astype(np.float64)
        near = False
        for c in range(1, T):
            p = O.tempered_probs(lg[tree.parent[c]], tau)
            th = min(eps, alpha * np.exp(-O.entropy(p)))
            if abs(p[tok[b, c]] - th) <= 1e-4 * th:
                near = True
        if near:
            skipped += 1
            continue
        n_acc, path, nxt, last = O.accept_typical(tree, tok[b], lg, tau, eps, alpha, None if u is None else float(u[b]))
        assert int(o.n_acc[b]) == n_acc and int(o.last_node[b]) == last
        assert o.path[b, :n_acc].tolist() == path and (o.path[b, n_acc:] == -1).all()
        lengths.add(n_acc)
        compared += 1
        if u is None:
            assert int(o.next_root[b]) == nxt
        else:
            cdf = np.cumsum(O.tempered_probs(lg[last], tau))
            if np.min(np.abs(cdf - float(u[b]))) > 1e-5:
                assert int(o.next_root[b]) == nxt
                sampled += 1
    print(f"{tree_name} V={V}: {compared} rows compared ({skipped} near-threshold rows skipped), accepted lengths {sorted(lengths)}, "
          f"{sampled} sampled tokens compared", flush=True)
    assert compared >= B - 1


def test_small_temperature_equals_accept_greedy_on_the_gpu():
    """tau -> 0 turns the criterion into greedy acceptance: both calls must return the same integers."""
    parent = frozen_tree("prior64")
    tree = O.Tree(parent)
    B, V, T = 4, 1000, tree.T
    sess, cfg = _session(parent, B, V)
    rng = np.random.default_rng(2)
    logits = rng.standard_normal((B, T, V)).astype(np.float32)
    amax = logits.argmax(-1)
    tok = rng.integers(0, V, size=(B, T))
    for b in range(B):
        for n in range(T):
            if tree.children[n] and rng.random() < 0.8:
                tok[b, tree.children[n][int(rng.integers(len(tree.children[n])))]] = amax[b, n]
    o = sess.out()
    o.tree_tokens.copy_(torch.tensor(tok, dtype=torch.int32)); o.logits.copy_(torch.tensor(logits))
    o.argmax.copy_(torch.tensor(amax, dtype=torch.int32))
    sess.main.accept_greedy(B, o.tree_tokens, o.argmax, o.n_acc, o.path, o.next_root, o.last_node)
    g = (o.n_acc.clone(), o.path.clone(), o.next_root.clone(), o.last_node.clone())
    sess.main.accept_typical(B, sess.ws, o.tree_tokens, o.logits, 1e-3, 0.3, 0.5, None, o.n_acc, o.path, o.next_root, o.last_node)
    torch.cuda.synchronize()
    assert torch.equal(o.n_acc, g[0]) and torch.equal(o.path, g[1]) and torch.equal(o.next_root, g[2]) and torch.equal(o.last_node, g[3])
    assert int(g[0].max()) >= 3


def test_accept_typical_argument_checks():
    from paper_2402_05109_amd import binding as hb
    sess, cfg = _session(frozen_tree("tiny16"), 1, 300)
    o = sess.out()
    for bad in ((0.0, 0.1, 0.3), (-1.0, 0.1, 0.3), (0.7, -0.1, 0.3), (0.7, 0.1, -1.0)):
        with pytest.raises(hb.HydraError) as e:
            sess.main.accept_typical(1, sess.ws, o.tree_tokens, o.logits, bad[0], bad[1], bad[2], None, o.n_acc, o.path, o.next_root, o.last_node)
        assert e.value.code == hb.E_INVALID_ARG
