"""GPU parity over seeded random shapes of the 16-bit family: widths that are not powers of two (d = 384, 640;
3 or 5 heads; F = 640, 896; ragged V), both head sizes, random trees of 1..128 nodes, 1..3 rows with different
lengths, shuffled page tables, 1..3-layer draft heads.  One draft + verify step each against the float64 oracle.

Tolerance 2e-2 (max relative error per row); ids exact outside counted near-ties.
"""
import numpy as np
import pytest
import torch

from oracle import hydra_oracle as O
from synth import uniform_tokens
from synth.trees import build_prior_tree
from helpers import make_weights, oracle_model, small_shape
from gpu_util import VerifyAudit, gpu_session, load_oracle_cache, max_rel, read_cache, to_np

pytestmark = pytest.mark.gpu
TOL = 2e-2


def _case(seed):
    r = np.random.default_rng(seed)
    Dh = int(r.choice([64, 128]))
    H = int(r.choice([2, 3, 5]))
    d = H * Dh
    if d % 128:
        H += 1; d = H * Dh                                   # the 16-bit family needs d % 128 == 0
    F = int(r.choice([384, 640, 896]))
    V = int(r.choice([257, 1000, 1531]))
    K = int(r.integers(1, 5))
    T = int(r.integers(1, 129))
    caps = tuple(int(r.integers(2, 9)) for _ in range(K))
    cap_nodes = 1
    tot = 1
    for c in caps:
        cap_nodes *= c; tot += cap_nodes
    T = min(T, tot)
    return dict(Dh=Dh, H=H, d=d, F=F, V=V, K=K, T=T, caps=caps, B=int(r.integers(1, 4)), mlp=int(r.integers(1, 4)),
                NL=int(r.integers(1, 3)), lens=[int(x) for x in r.integers(0, 300, size=3)])


@pytest.mark.parametrize("seed", list(range(10)))
def test_random_shape_draft_and_verify(seed):
    c = _case(seed)
    print("case", c, flush=True)
    cfg = small_shape(dtype="bf16", d=c["d"], NL=c["NL"], H=c["H"], Dh=c["Dh"], F=c["F"], V=c["V"], K=c["K"], mlp_layers=c["mlp"], T=c["T"])
    W = make_weights(cfg, gain_std=0.1, std=0.05)
    parent = build_prior_tree(c["T"], c["caps"])
    tree = O.Tree(parent)
    T, B = tree.T, c["B"]
    lens = c["lens"][:B]
    Lmax = max(lens)
    m = oracle_model(cfg, W)
    sess = gpu_session(cfg, parent, B, Lmax + 16, W, page_perm_seed=seed, want_logits=True)
    rng = np.random.default_rng(1000 + seed)
    h16 = lambda a: torch.tensor(a, dtype=torch.float32).to(torch.float16).double().numpy()
    caches = []
    for b in range(B):
        cch = O.FlatCache(m, Lmax + T)
        cch.K[:, :lens[b]] = h16(rng.standard_normal(cch.K[:, :lens[b]].shape))
        cch.V[:, :lens[b]] = h16(rng.standard_normal(cch.V[:, :lens[b]].shape))
        caches.append(cch)
    load_oracle_cache(sess, caches, Lmax)
    sess.seq_len.copy_(torch.tensor(lens, dtype=torch.int32)); sess.host_len = Lmax
    # draft
    h = rng.standard_normal((B, cfg.d)).astype(np.float32)
    roots = [int(t) for t in uniform_tokens(seed, 7, B, cfg.V)]
    sess.h_last.copy_(torch.tensor(h)); sess.root.copy_(torch.tensor(roots, dtype=torch.int32))
    sess.draft()
    torch.cuda.synchronize()
    o = sess.out()
    exact = audited = 0
    for b in range(B):
        got = o.tree_tokens[b].cpu().tolist()
        assert got[0] == roots[b]
        _, lg = O.draft_tree(m, tree, h[b].astype(np.float64), roots[b], forced_tokens=got)
        for n, logits in lg.items():
            kids = [got[ch] for ch in tree.children[n]]
            ref = O.top_k_ids(logits, len(kids))
            if kids == ref:
                exact += 1
                continue
            audited += 1
            tol = TOL * np.max(np.abs(logits))
            vals = logits[kids]
            assert len(set(kids)) == len(kids) and np.all(np.diff(vals) <= tol) and vals[-1] >= logits[ref[-1]] - tol
    assert exact >= audited
    # verify
    toks = np.stack([uniform_tokens(seed, 50 + b, T, cfg.V).numpy() for b in range(B)])
    o.tree_tokens.copy_(torch.tensor(toks, dtype=torch.int32))
    sess.verify()
    torch.cuda.synchronize()
    assert sess.main.read_flags() == 0
    audit = VerifyAudit(TOL)
    for b in range(B):
        L = lens[b]
        hid, logits, amax = O.tree_verify(m, caches[b], L, tree, toks[b].tolist())
        assert max_rel(to_np(o.hidden[b]), hid) <= TOL and max_rel(to_np(o.logits[b]), logits) <= TOL
        audit.add(o.logits[b].cpu().numpy(), o.argmax[b].cpu().numpy(), o.margin[b].cpu().numpy(), logits, amax)
        for l in range(cfg.NL):
            t = torch.zeros(B, T, 2, cfg.H, cfg.Dh, dtype=torch.float32, device="cuda:0")
            sess.main.kv_read(B, l, sess.kv, L, T, t)
            kv = to_np(t[b])
            assert max_rel(kv[:, 0].reshape(T, -1), caches[b].K[l, L:L + T].reshape(T, -1)) <= TOL
            assert max_rel(kv[:, 1].reshape(T, -1), caches[b].V[l, L:L + T].reshape(T, -1)) <= TOL
    print(f"seed {seed}: draft {exact} exact / {audited} audited", flush=True)
    audit.finish(f"seed {seed}", max_skip_frac=0.3)
