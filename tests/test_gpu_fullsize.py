"""GPU parity at the benchmark's full width: the 7B shape of the headline
workload (d = 4096, 32 heads x 128, FFN 11008, V = 32000, 64-node tree, B = 1,
4 draft heads), in the launch configuration bench.py times, with the number of
decoder layers cut to 2 so that the float64 oracle finishes in well under a
minute.  Every kernel shape of the 32-layer run appears here (the per-layer
GEMMs, the LM head, the four head sizes, tree attention at a ragged context of
several hundred tokens).  The KV cache content is seeded synthetic data written
through hydra_kv_write, not a prefill: parity of one step holds for any cache.

Tolerance as everywhere for bf16: max relative error per row 2e-2; ids exact
unless the oracle's own top-2 margin is inside that tolerance (counted).
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


@pytest.fixture(scope="module")
def full():
    from paper_2402_05109_amd.session import Session
    cfg = CONFIGS[2].with_(NL=2)
    spec = WeightSpec(cfg, gain_std=0.1)
    names = tensor_names(cfg)
    dev = "cuda:0"
    W = {}
    for n in names:                                   # generated on the device, kept on the host for the oracle
        W[n] = make_tensor(spec, n, device=dev).cpu()
    parent = frozen_tree("prior64")
    L = 523                                           # ragged: 32 full key tiles + 11, then the 64 tree slots
    sess = Session(cfg, parent, 1, L + 64, lambda n: W[n].to(dev), prefill_chunk=64, want_logits=True)
    m = oracle_model(cfg, W, keep=True)
    return cfg, W, parent, L, sess, m


def test_generator_is_bit_identical_on_cpu_and_gpu(full):
    cfg, W, *_ = full
    spec = WeightSpec(cfg, gain_std=0.1)
    for n in ("layers.1.wq", "heads.2.b1", "final_norm"):
        assert torch.equal(make_tensor(spec, n, device="cpu"), W[n])


def test_tree_verify_forward_full_width(full):
    cfg, W, parent, L, sess, m = full
    tree = O.Tree(parent)
    T = tree.T
    rng = np.random.default_rng(7)
    cache = O.FlatCache(m, L + T)
    bf = lambda a: torch.tensor(a, dtype=torch.float32).to(torch.float16).double().numpy()    # exactly what the cache holds
    cache.K[:, :L] = bf(rng.standard_normal(cache.K[:, :L].shape) * 0.5)
    cache.V[:, :L] = bf(rng.standard_normal(cache.V[:, :L].shape) * 0.5)
    load_oracle_cache(sess, [cache], L)
    toks = uniform_tokens(99, 0, T, cfg.V).tolist()
    o = sess.out()
    o.tree_tokens.copy_(torch.tensor([toks], dtype=torch.int32))
    sess.verify()
    torch.cuda.synchronize()
    assert sess.main.read_flags() == 0
    hid, logits, amax = O.tree_verify(m, cache, L, tree, toks)
    eh = max_rel(to_np(o.hidden[0]), hid)
    audit = VerifyAudit(TOL)
    audit.add(o.logits[0].cpu().numpy(), o.argmax[0].cpu().numpy(), o.margin[0].cpu().numpy(), logits, amax)
    el, skipped = audit.finish("full width, 2 layers", max_skip_frac=0.2)
    newkv = read_cache(sess, sess.main, L, T)
    ek = max(max_rel(newkv[l, 0, :, 0].reshape(T, -1), cache.K[l, L:L + T].reshape(T, -1)) for l in range(cfg.NL))
    ev = max(max_rel(newkv[l, 0, :, 1].reshape(T, -1), cache.V[l, L:L + T].reshape(T, -1)) for l in range(cfg.NL))
    print(f"full width: hidden err {eh:.4f} logits err {el:.4f} K err {ek:.4f} V err {ev:.4f}; "
          f"argmax exact on {T - skipped} rows, {skipped} near-tie rows", flush=True)
    assert eh <= TOL and el <= TOL and ek <= TOL and ev <= TOL


def test_draft_tree_full_width(full):
    cfg, W, parent, L, sess, m = full
    tree = O.Tree(parent)
    rng = np.random.default_rng(8)
    h = rng.standard_normal(cfg.d).astype(np.float32)
    sess.h_last.copy_(torch.tensor(h).reshape(1, -1))
    sess.root.fill_(1234)
    sess.draft()
    torch.cuda.synchronize()
    got = sess.out().tree_tokens[0].cpu().tolist()
    assert got[0] == 1234
    _, lg = O.draft_tree(m, tree, h.astype(np.float64), 1234, forced_tokens=got)
    exact = audited = 0
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
    print(f"full width draft: {exact} nodes exact, {audited} with near-tie reorderings", flush=True)
    assert exact >= audited
    assert sess.main.read_flags() == 0


def test_step_integer_tail_full_width(full):
    """accept + compact after the verify above: integer outputs against the oracle fed with the GPU's
    own tokens and argmax (bit-exact), and the moved cache bytes."""
    cfg, W, parent, L, sess, m = full
    tree = O.Tree(parent)
    o = sess.out()
    rng = np.random.default_rng(9)
    tok = rng.integers(0, cfg.V, size=tree.T)
    amax = rng.integers(0, cfg.V, size=tree.T)
    cur = 0
    for depth in range(3):                                # plant an accepted path of length 4
        c = tree.children[cur][min(1, len(tree.children[cur]) - 1)]
        amax[cur] = tok[c]
        cur = c
    o.tree_tokens.copy_(torch.tensor(tok.reshape(1, -1), dtype=torch.int32))
    o.argmax.copy_(torch.tensor(amax.reshape(1, -1), dtype=torch.int32))
    sess.seq_len.fill_(L); sess.host_len = L
    before = read_cache(sess, sess.main, L, tree.T)
    sess.accept(); sess.compact()
    torch.cuda.synchronize()
    n_acc, path, nxt, last = O.accept_greedy(tree, tok, amax)
    assert n_acc == 4
    assert int(o.n_acc[0]) == n_acc and o.path[0, :n_acc].tolist() == path and int(o.next_root[0]) == nxt
    assert int(sess.seq_len[0]) == L + n_acc and int(sess.root[0]) == nxt
    after = read_cache(sess, sess.main, L, tree.T)
    for j, n in enumerate(path):
        np.testing.assert_array_equal(after[:, 0, j], before[:, 0, n])
    pt = sess.page_table.cpu().numpy()
    for j in range(n_acc):
        assert o.kv_index[0, j].tolist() == [int(pt[0, (L + j) // 16]), (L + j) % 16]
    assert torch.equal(sess.h_last[0], o.hidden[0, last])


def test_tree_verify_forward_full_depth_32_layers():
    """The headline workload itself: all 32 layers of the 7B shape, T = 64, B = 1, context 523, one verify
    step against the float64 oracle (about 10 s of CPU).  This is where rounding accumulates: the bound
    is still the 2e-2 of the 2-layer cases."""
    from paper_2402_05109_amd.session import Session
    cfg = CONFIGS[2].with_(K=1)                       # the draft heads are covered above; keep host memory small
    spec = WeightSpec(cfg)
    dev = "cuda:0"
    W = {n: make_tensor(spec, n, device=dev).cpu() for n in tensor_names(cfg)}
    parent = frozen_tree("prior64")
    tree = O.Tree(parent)
    T, L = tree.T, 523
    sess = Session(cfg, parent, 1, L + 64, lambda n: W[n].to(dev), prefill_chunk=64, want_logits=True)
    m = oracle_model(cfg, W, keep=False)
    rng = np.random.default_rng(7)
    cache = O.FlatCache(m, L + T)
    h16 = lambda a: torch.tensor(a, dtype=torch.float32).to(torch.float16).double().numpy()
    cache.K[:, :L] = h16(rng.standard_normal(cache.K[:, :L].shape) * 0.5)
    cache.V[:, :L] = h16(rng.standard_normal(cache.V[:, :L].shape) * 0.5)
    load_oracle_cache(sess, [cache], L)
    toks = uniform_tokens(99, 0, T, cfg.V).tolist()
    o = sess.out()
    o.tree_tokens.copy_(torch.tensor([toks], dtype=torch.int32))
    sess.verify()
    torch.cuda.synchronize()
    assert sess.main.read_flags() == 0
    print("GPU verify done, oracle running", flush=True)
    hid, logits, amax = O.tree_verify(m, cache, L, tree, toks)
    eh = max_rel(to_np(o.hidden[0]), hid)
    audit = VerifyAudit(TOL)
    audit.add(o.logits[0].cpu().numpy(), o.argmax[0].cpu().numpy(), o.margin[0].cpu().numpy(), logits, amax)
    # the near-tie threshold follows the error measured here, which after 32 layers is about four times that of the
    # 2-layer cases: with random-init logits over 32000 ids roughly a third of the rows then lie under it
    el, skipped = audit.finish("full width, 32 layers", max_skip_frac=0.5)
    print(f"32 layers: hidden err {eh:.4f} logits err {el:.4f}; argmax exact on {T - skipped} rows, {skipped} near-tie rows", flush=True)
    assert eh <= TOL and el <= TOL
