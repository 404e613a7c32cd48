"""GPU parity of hydra_draft_tree with Medusa-style heads (paper, section 2: p_draft = f_draft,i(h_{t-1}), one
hidden layer with a skip connection; section 3: no sequential dependence) against the oracle.

fp32 family: drafted ids exact.  16-bit family: ids exact or a valid reordering inside the 2e-2 tolerance
(counted).  On both the drafted lists must not depend on the candidate path.
"""
import numpy as np
import pytest
import torch

from oracle import hydra_oracle as O
from synth import frozen_tree, uniform_tokens
from helpers import make_weights, oracle_model, small_shape
from gpu_util import gpu_session

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype,mlp,tree_name,B", [("f32", 1, "tiny16", 3), ("f32", 3, "prior32", 1), ("bf16", 1, "prior64", 2),
                                                   ("bf16", 4, "tiny16", 4)])
def test_medusa_draft_matches_oracle(dtype, mlp, tree_name, B):
    if dtype == "f32":
        cfg, tol = small_shape(medusa=1, d=128, NL=1, H=2, Dh=64, F=176, V=300, K=4, mlp_layers=mlp), 1e-4
    else:
        cfg, tol = small_shape(medusa=1, dtype="bf16", d=256, NL=1, H=2, Dh=128, F=384, V=1000, K=4, mlp_layers=mlp), 2e-2
    W = make_weights(cfg, std=0.06)
    parent = frozen_tree(tree_name)
    tree = O.Tree(parent)
    m = oracle_model(cfg, W)
    sess = gpu_session(cfg, parent, B, 32, W)
    rng = np.random.default_rng(12)
    h = rng.standard_normal((B, cfg.d)).astype(np.float32)
    roots = uniform_tokens(5, 0, B, cfg.V)
    sess.h_last.copy_(torch.tensor(h)); sess.root.copy_(roots)
    sess.draft()
    torch.cuda.synchronize()
    assert sess.main.read_flags() == 0
    got = sess.out().tree_tokens.cpu().tolist()
    exact = audited = 0
    for b in range(B):
        assert got[b][0] == int(roots[b])
        want, lg = O.draft_tree(m, tree, h[b].astype(np.float64), int(roots[b]))
        for n, logits in lg.items():
            kids = [got[b][c] for c in tree.children[n]]
            ref = O.top_k_ids(logits, len(kids))
            if kids == ref:
                exact += 1
                continue
            assert dtype == "bf16", "fp32 family: ids must be exact"
            audited += 1
            t = tol * np.max(np.abs(logits))
            vals = logits[kids]
            assert len(set(kids)) == len(kids) and np.all(np.diff(vals) <= t) and vals[-1] >= logits[ref[-1]] - t
        # path independence on the device: nodes of one depth hold prefixes of one list
        for i in range(1, tree.max_depth + 1):
            lists = [[got[b][c] for c in tree.children[n]] for n in range(tree.T) if tree.depth[n] == i - 1 and tree.children[n]]
            longest = max(lists, key=len)
            assert all(l == longest[:len(l)] for l in lists)
    print(f"{dtype} mlp={mlp} {tree_name}: {exact} nodes exact, {audited} audited", flush=True)
    assert exact >= audited
