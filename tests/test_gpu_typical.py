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


def _near_threshold_or_cdf_step(tree, tok, logits, tau, eps, alpha, u, last):
    """True if float32 could decide this step differently from float64: some candidate's probability within 1e-4
    (relative) of its threshold, or u within 1e-5 of a step of the cumulative distribution at the last node."""
    for c in range(1, tree.T):
        p = O.tempered_probs(logits[tree.parent[c]], tau)
        th = min(eps, alpha * np.exp(-O.entropy(p)))
        if abs(p[tok[c]] - th) <= 1e-4 * th:
            return True
    cdf = np.cumsum(O.tempered_probs(logits[last], tau))
    return bool(np.min(np.abs(cdf - u)) <= 1e-5)


@pytest.mark.parametrize("prefix", [0, 1])
def test_typical_acceptance_loop_matches_the_oracle_token_for_token(prefix):
    """Section 6.3 as the criterion of the whole loop, fp32 tiny configuration, free running: draft -> verify ->
    accept_typical (next root drawn at supplied uniform numbers) -> kv_compact (-> prefix layer), 32 tokens, against
    the oracle's loop with the same numbers: emitted tokens, acceptance lengths and drawn roots, step by step, until
    the first step whose decision float32 could take differently (counted; none is expected at this size)."""
    from synth import CONFIGS, uniform_tokens
    from helpers import oracle_model
    cfg = CONFIGS[1].with_(prefix=prefix)
    W = make_weights(cfg, gain_std=0.0)
    m = oracle_model(cfg, W)
    parent = frozen_tree("tiny16")
    tree = O.Tree(parent)
    prompt = uniform_tokens(cfg.seed, 0, 48, cfg.V)
    # random-init logits are nearly flat (p about 1/V, exp(-H) about 1/V): with alpha = 1 a candidate passes iff its
    # logit is above a tempered average, about every second one, so paths of all lengths occur
    tau, eps, alpha = 1.0, 0.5, 1.0
    us = np.random.default_rng(12).random(64).astype(np.float32)
    log = []
    want, want_acc = O.hydra_generate(m, tree, prompt.tolist(), 32, prefix=bool(prefix), typical=(tau, eps, alpha),
                                      u_per_step=us.astype(np.float64), step_log=log)
    sess = gpu_session(cfg, parent, 1, 48 + 32 + 24, W, prefill_chunk=16, want_logits=True)
    sess.prefill(prompt.reshape(1, -1))
    o = sess.out()
    emitted, compared = [], 0
    for s, info in enumerate(log):
        ud = torch.tensor(us[s:s + 1], device="cuda:0")
        sess.step(typical=(tau, eps, alpha, ud))
        torch.cuda.synchronize()
        assert sess.main.read_flags() == 0
        na = int(o.n_acc[0])
        got_path = o.path[0, :na].tolist()
        risky = _near_threshold_or_cdf_step(tree, info["tok"], info["logits"], tau, eps, alpha, float(us[s]), info["path"][-1])
        same = (o.tree_tokens[0].tolist() == info["tok"] and got_path == info["path"] and int(o.next_root[0]) == info["next_root"])
        if not same:
            assert risky, f"step {s}: the library and the oracle differ away from a threshold"
            break
        emitted += [info["tok"][n] for n in got_path]
        compared += 1
        sess.sync_len()
    print(f"typical loop (prefix={prefix}): {compared} of {len(log)} steps compared, acceptance lengths {want_acc[:compared]}", flush=True)
    assert compared >= len(log) - 1 and len(set(want_acc[:compared])) >= 3
    assert emitted[:32] == want[:len(emitted[:32])]


def test_typical_acceptance_step_in_the_16_bit_family_teacher_forced():
    """One step of the 16-bit family with the library's own logits: accept_typical's integers must equal the oracle's
    criterion evaluated on those very logits (rows near a threshold excluded and counted), and kv_compact must then
    advance the state along that path."""
    from test_gpu_bf16 import bf16_shape
    cfg = bf16_shape()
    W = make_weights(cfg, gain_std=0.1, std=0.05)
    parent = frozen_tree("prior64")
    tree = O.Tree(parent)
    B, T, L = 3, tree.T, 40
    sess = gpu_session(cfg, parent, B, 128, W, want_logits=True, page_perm_seed=4)
    rng = np.random.default_rng(5)
    for l in range(cfg.NL):
        t = torch.tensor(rng.standard_normal((B, L, 2, cfg.H, cfg.Dh)) * 0.5, dtype=torch.float32, device="cuda:0")
        sess.main.kv_write(B, l, sess.kv, 0, L, t)
    sess.seq_len.fill_(L); sess.host_len = L
    o = sess.out()
    from synth import uniform_tokens
    o.tree_tokens.copy_(torch.stack([uniform_tokens(9, b, T, cfg.V) for b in range(B)]).to(torch.int32))
    sess.verify()
    tau, eps, alpha = 3.0, 0.5, 0.9
    u = torch.tensor(rng.random(B).astype(np.float32), device="cuda:0")
    sess.accept_typical(tau, eps, alpha, u)
    sess.compact()
    torch.cuda.synchronize()
    assert sess.main.read_flags() == 0
    tok = o.tree_tokens.cpu().numpy(); lg = o.logits.cpu().numpy().astype(np.float64)
    compared = 0
    for b in range(B):
        n_acc, path, nxt, last = O.accept_typical(tree, tok[b], lg[b], tau, eps, alpha, float(u[b]))
        if _near_threshold_or_cdf_step(tree, tok[b], lg[b], tau, eps, alpha, float(u[b]), last):
            continue
        compared += 1
        assert int(o.n_acc[b]) == n_acc and o.path[b, :n_acc].tolist() == path and int(o.next_root[b]) == nxt
        assert int(sess.seq_len[b]) == L + n_acc and int(sess.root[b]) == nxt
        assert torch.equal(sess.h_last[b], o.hidden[b, last])
    print("16-bit typical step: rows compared", compared, "lengths", o.n_acc.tolist(), flush=True)
    assert compared >= B - 1 and int(o.n_acc.max()) >= 2
