"""GPU parity at the widths of the other workload configurations: the 7B shape with
Hydra++ heads (4-layer MLPs) at batch 4, 8 and 16, the 13B shape (also at its longest prompt,
4096) and the 33B shape (trees of 32, 64 and 128 nodes, batch 1 and 4).  Each
runs one draft + verify step at full width against the float64 oracle with the
number of decoder layers (and, for the 33B shape, of draft heads) cut so that the
oracle needs about ten seconds and a few GB; widths, head counts, FFN sizes,
vocabulary, tree and batch are the configuration's own.  The KV cache content is
seeded synthetic data written through hydra_kv_write.

Tolerance as everywhere for the bf16 family: max relative error per row 2e-2; ids
exact unless the oracle's top-2 margin is inside the tolerance (counted).
"""
import numpy as np
import pytest
import torch

from oracle import hydra_oracle as O
from synth import CONFIGS, WeightSpec, frozen_tree, make_tensor, tensor_names, uniform_tokens
from helpers import oracle_model
from gpu_util import VerifyAudit, load_oracle_cache, max_rel, read_cache, to_np

pytestmark = pytest.mark.gpu
TOL = 2e-2

CASES = [
    # config, overrides, batch, context per row
    pytest.param(3, dict(NL=2), 4, (301, 17, 256, 90), id="config3-7b-hydra++-batch4"),
    pytest.param(4, dict(NL=1), 1, (523,), id="config4-13b"),
    pytest.param(5, dict(NL=1, K=2), 1, (210,), id="config5-33b"),
    # config 5's other tree sizes and its batch of 4 (128 rows per GEMM in both)
    pytest.param(5, dict(NL=1, K=2, tree="prior128"), 1, (333,), id="config5-33b-tree128"),
    pytest.param(5, dict(NL=1, K=2, tree="prior32"), 4, (97, 2048, 640, 15), id="config5-33b-tree32-batch4"),
    # config 4's longest prompt: the keys of a head are split over workgroups and merged, at 40 heads
    pytest.param(4, dict(NL=1), 1, (4096,), id="config4-13b-context4096"),
    # 512 and 1024 rows per GEMM: the many-rows kernel that shares the X tiles through LDS (four and eight waves)
    pytest.param(3, dict(NL=1), 8, (70, 3, 129, 16, 200, 64, 31, 150), id="config3-7b-hydra++-batch8"),
    pytest.param(3, dict(NL=1), 16, (40, 3, 129, 16, 100, 64, 31, 90, 1, 77, 128, 5, 60, 33, 17, 111), id="config3-7b-hydra++-batch16"),
]


@pytest.mark.parametrize("idx,over,B,lens", CASES)
def test_draft_and_verify_at_full_width(idx, over, B, lens):
    from paper_2402_05109_amd.session import Session
    over = dict(over)
    tree_name = over.pop("tree", "prior64")
    cfg = CONFIGS[idx].with_(**over)
    spec = WeightSpec(cfg, gain_std=0.1)
    dev = "cuda:0"
    W = {n: make_tensor(spec, n, device=dev).cpu() for n in tensor_names(cfg)}
    parent = frozen_tree(tree_name)
    if cfg.K < 4:                                       # fewer heads: cut the tree at depth K
        depth = [0] * len(parent)
        for n in range(1, len(parent)):
            depth[n] = depth[parent[n]] + 1
        keep = [n for n in range(len(parent)) if depth[n] <= cfg.K]
        assert keep == list(range(len(keep)))           # breadth-first order: a prefix
        parent = parent[:len(keep)]
    tree = O.Tree(parent)
    T = tree.T
    Lmax = max(lens)
    sess = Session(cfg, parent, B, Lmax + 64, lambda n: W[n].to(dev), prefill_chunk=64, want_logits=True)
    m = oracle_model(cfg, W, keep=True)                 # float64 copies are kept: up to ~15 GB of host memory for the 33B width
    rng = np.random.default_rng(100 + idx)
    h16 = lambda a: torch.tensor(a, dtype=torch.float32).to(torch.float16).double().numpy()
    caches = []
    for b in range(B):
        c = O.FlatCache(m, Lmax + T)
        c.K[:, :lens[b]] = h16(rng.standard_normal(c.K[:, :lens[b]].shape) * 0.5)
        c.V[:, :lens[b]] = h16(rng.standard_normal(c.V[:, :lens[b]].shape) * 0.5)
        caches.append(c)
    load_oracle_cache(sess, caches, Lmax)               # slots past a row's own length hold zeros and are never visible
    sess.seq_len.copy_(torch.tensor(lens, dtype=torch.int32))
    sess.host_len = Lmax

    # ---- draft: the library's tree, audited node by node against the oracle fed with the same path tokens
    h = rng.standard_normal((B, cfg.d)).astype(np.float32)
    roots = [int(t) for t in uniform_tokens(7, idx, B, cfg.V)]
    sess.h_last.copy_(torch.tensor(h))
    sess.root.copy_(torch.tensor(roots, dtype=torch.int32))
    sess.draft()
    torch.cuda.synchronize()
    o = sess.out()
    exact = audited = 0
    for b in range(B):
        got = o.tree_tokens[b].cpu().tolist()
        assert got[0] == roots[b]
        _, lg = O.draft_tree(m, tree, h[b].astype(np.float64), roots[b], forced_tokens=got)
        for n, logits in lg.items():
            kids = [got[c] for c in tree.children[n]]
            ref = O.top_k_ids(logits, len(kids))
            if kids == ref:
                exact += 1
                continue
            audited += 1
            tol = TOL * np.max(np.abs(logits))
            vals = logits[kids]
            assert len(set(kids)) == len(kids)
            assert np.all(np.diff(vals) <= tol) and vals[-1] >= logits[ref[-1]] - tol
    assert exact >= audited

    # ---- verify on seeded tokens
    toks = np.stack([uniform_tokens(99, b, T, cfg.V).numpy() for b in range(B)])
    o.tree_tokens.copy_(torch.tensor(toks, dtype=torch.int32))
    sess.verify()
    torch.cuda.synchronize()
    assert sess.main.read_flags() == 0
    worst = dict(h=0.0, l=0.0, k=0.0, v=0.0)
    audit = VerifyAudit(TOL)
    for b in range(B):
        L = lens[b]
        hid, logits, amax = O.tree_verify(m, caches[b], L, tree, toks[b].tolist())
        worst["h"] = max(worst["h"], max_rel(to_np(o.hidden[b]), hid))
        worst["l"] = max(worst["l"], max_rel(to_np(o.logits[b]), logits))
        audit.add(o.logits[b].cpu().numpy(), o.argmax[b].cpu().numpy(), o.margin[b].cpu().numpy(), logits, amax)
        for l in range(cfg.NL):
            t = torch.zeros(B, T, 2, cfg.H, cfg.Dh, dtype=torch.float32, device=dev)
            sess.main.kv_read(B, l, sess.kv, L, T, t)
            kv = to_np(t[b])
            worst["k"] = max(worst["k"], max_rel(kv[:, 0].reshape(T, -1), caches[b].K[l, L:L + T].reshape(T, -1)))
            worst["v"] = max(worst["v"], max_rel(kv[:, 1].reshape(T, -1), caches[b].V[l, L:L + T].reshape(T, -1)))
    # ---- Hydra++ prefix attention on a scripted accepted path (left-most chain, length varying with the row)
    rngp = np.random.default_rng(200 + idx)
    pcs = []
    pctx = sess.prefix_ctx(tree.max_depth + 1)
    plain = np.zeros((B, Lmax, 2, cfg.H, cfg.Dh))
    for b in range(B):
        pc = O.PrefixCache(m, Lmax + T)
        pc.K[:lens[b]] = h16(rngp.standard_normal(pc.K[:lens[b]].shape) * 0.5)
        pc.V[:lens[b]] = h16(rngp.standard_normal(pc.V[:lens[b]].shape) * 0.5)
        plain[b, :, 0], plain[b, :, 1] = pc.K[:Lmax], pc.V[:Lmax]
        pcs.append(pc)
    pctx.kv_write(B, 0, sess.pkv, 0, Lmax, torch.tensor(plain, dtype=torch.float32, device=dev).contiguous())
    sess.pseq_len.copy_(torch.tensor(lens, dtype=torch.int32))
    chain = [0]
    while tree.children[chain[-1]]:
        chain.append(tree.children[chain[-1]][0])
    n_accs = [1 + (b + idx) % len(chain) for b in range(B)]
    path = np.full((B, tree.max_depth + 1), -1, dtype=np.int32)
    for b in range(B):
        path[b, :n_accs[b]] = chain[:n_accs[b]]
    o.path.copy_(torch.tensor(path)); o.n_acc.copy_(torch.tensor(n_accs, dtype=torch.int32))
    hid_gpu = to_np(o.hidden)                           # the layer's input is the library's own verify output
    sess.host_len = Lmax
    sess.prefix_attention()
    torch.cuda.synchronize()
    assert pctx.read_flags() == 0
    assert sess.pseq_len.tolist() == [lens[b] + n_accs[b] for b in range(B)]
    worst_p = 0.0
    for b in range(B):
        for j in range(n_accs[b]):
            g = O.prefix_token(m, pcs[b], hid_gpu[b, chain[j]], lens[b] + j)
        worst_p = max(worst_p, max_rel(to_np(sess.h_last[b]), g))
        t = torch.zeros(B, n_accs[b], 2, cfg.H, cfg.Dh, dtype=torch.float32, device=dev)
        pctx.kv_read(B, 0, sess.pkv, lens[b], n_accs[b], t)
        kvp = to_np(t[b])
        worst_p = max(worst_p, max_rel(kvp[:, 0].reshape(n_accs[b], -1), pcs[b].K[lens[b]:lens[b] + n_accs[b]].reshape(n_accs[b], -1)))
        worst_p = max(worst_p, max_rel(kvp[:, 1].reshape(n_accs[b], -1), pcs[b].V[lens[b]:lens[b] + n_accs[b]].reshape(n_accs[b], -1)))
    print(f"config {idx}: prefix attention, accepted lengths {n_accs}: worst error {worst_p:.4f}", flush=True)
    assert worst_p <= TOL

    print(f"config {idx} {over} B={B}: draft {exact} nodes exact / {audited} audited; verify hidden {worst['h']:.4f} "
          f"logits {worst['l']:.4f} K {worst['k']:.4f} V {worst['v']:.4f}", flush=True)
    assert max(worst.values()) <= TOL
    audit.finish(f"config {idx} B={B}", max_skip_frac=0.2)
