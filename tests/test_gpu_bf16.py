"""GPU parity, bf16 family (MFMA GEMM, MFMA tree attention) against the CPU oracle.

Tolerance: integer results bit-exact; floating point max relative error per row
<= 2e-2 (max|gpu - ref| / max|ref|).  An exact-id check is skipped, and counted,
where the oracle's own top-2 margin is below that tolerance; the id the GPU
picked must then still be within the tolerance of the oracle's maximum.
Shapes are small enough for the oracle to finish in seconds but span several
32-wide tiles, a ragged vocabulary (V = 1000) and ragged context lengths.
"""
import numpy as np
import pytest
import torch

from oracle import hydra_oracle as O
from synth import chain_tree, frozen_tree, proposal_trees, random_tree, star_tree, uniform_tokens
from helpers import make_weights, oracle_model, small_shape
from gpu_util import VerifyAudit, gpu_session, load_oracle_cache, max_rel, near_tie, read_cache, to_np

pytestmark = pytest.mark.gpu
TOL = 2e-2


def bf16_shape(**kw):
    base = dict(d=256, NL=2, H=2, Dh=128, F=384, V=1000, K=4, mlp_layers=1, dtype="bf16")
    base.update(kw)
    return small_shape(**base)


def bf16_round(a):
    return torch.tensor(a, dtype=torch.float32).to(torch.bfloat16).double().numpy()


def cache_round(a):
    """Values the 16-bit KV cache holds exactly (the library keeps them as IEEE half)."""
    return torch.tensor(a, dtype=torch.float32).to(torch.float16).double().numpy()


TREES = {"tiny16": lambda: frozen_tree("tiny16"), "prior64": lambda: frozen_tree("prior64"),
         "prior128": lambda: frozen_tree("prior128"), "prior32": lambda: frozen_tree("prior32"),
         "single": lambda: [-1], "chain40": lambda: chain_tree(40), "random70": lambda: random_tree(70, 4, 3),
         # proposal trees of the tree-size sweep (sizes that are none of the frozen workload trees)
         "sweep12": lambda: proposal_trees(12)[-1], "sweep24": lambda: proposal_trees(24)[-1], "sweep48": lambda: proposal_trees(48)[-1]}


@pytest.mark.parametrize("tree_name,L,B,Dh", [("prior64", 0, 1, 128), ("prior64", 1, 2, 128), ("prior64", 31, 1, 128),
                                               ("prior64", 32, 1, 128), ("prior64", 33, 2, 128), ("prior64", 500, 1, 128),
                                               ("tiny16", 17, 3, 128), ("prior128", 200, 1, 128), ("random70", 77, 2, 128),
                                               ("single", 129, 2, 128), ("chain40", 8, 1, 128), ("prior64", 95, 2, 64),
                                               ("prior32", 1000, 1, 128),
                                               # beyond ~1200 keys the keys of a head are split over workgroups and merged
                                               ("prior64", 1500, 1, 128), ("prior128", 1400, 2, 64), ("tiny16", 2500, 1, 128)])
def test_tree_attention_sharp_scores(tree_name, L, B, Dh):
    print("case", tree_name, L, B, Dh, flush=True)
    cfg = bf16_shape(H=256 // Dh, Dh=Dh)
    W = make_weights(cfg)
    parent = TREES[tree_name]()
    tree = O.Tree(parent)
    T = tree.T
    sess = gpu_session(cfg, parent, B, L + 64, W, page_perm_seed=5)
    rng = np.random.default_rng(200 + L)
    q = bf16_round(rng.standard_normal((B, T, cfg.H, cfg.Dh)) * 1.5)
    keys = bf16_round(rng.standard_normal((B, L + T, cfg.H, cfg.Dh)) * 1.5)
    vals = bf16_round(rng.standard_normal((B, L + T, cfg.H, cfg.Dh)))
    plain = torch.tensor(np.stack([keys, vals], axis=2), dtype=torch.float32, device="cuda:0").contiguous()
    layer = 1
    sess.main.kv_write(B, layer, sess.kv, 0, L + T, plain)
    sess.seq_len.fill_(L)
    out = torch.zeros(B, T, cfg.H, cfg.Dh, dtype=torch.float32, device="cuda:0")
    qd = torch.tensor(q, dtype=torch.float32, device="cuda:0").contiguous()
    for hint in (0, L):
        sess.kv.seq_len_hint = hint
        out.zero_()
        sess.main.tree_attention(B, layer, sess.ws, qd, sess.seq_len, sess.kv, out)
        torch.cuda.synchronize()
        got = to_np(out)
        worst = 0.0
        for b in range(B):
            for h in range(cfg.H):
                ref = O.tree_attention(q[b, :, h], keys[b, :, h], vals[b, :, h], L, tree)
                worst = max(worst, max_rel(got[b, :, h], ref))
        print("hint", hint, "max rel err", worst, flush=True)
        assert worst <= TOL
    assert sess.main.read_flags() == 0


def test_tree_attention_one_hot_values_name_the_keys():
    cfg = bf16_shape()
    W = make_weights(cfg)
    parent = frozen_tree("prior64")
    tree = O.Tree(parent)
    T, L = tree.T, 50
    assert L + T <= cfg.Dh
    sess = gpu_session(cfg, parent, 1, 128, W)
    vals = np.zeros((1, L + T, cfg.H, cfg.Dh)); keys = np.zeros_like(vals)
    for s in range(L + T):
        vals[0, s, :, s] = 1.0
    plain = torch.tensor(np.stack([keys, vals], axis=2), dtype=torch.float32, device="cuda:0").contiguous()
    sess.main.kv_write(1, 0, sess.kv, 0, L + T, plain)
    sess.seq_len.fill_(L)
    q = torch.zeros(1, T, cfg.H, cfg.Dh, dtype=torch.float32, device="cuda:0")
    out = torch.zeros_like(q)
    sess.main.tree_attention(1, 0, sess.ws, q, sess.seq_len, sess.kv, out)
    got = to_np(out)[0]
    for n in range(T):
        seen = set(range(L)) | {L + a for a in tree.path(n)}
        row = np.zeros(cfg.Dh); row[list(seen)] = 1.0 / len(seen)
        for h in range(cfg.H):
            np.testing.assert_allclose(got[n, h], row, atol=2e-4)      # 1/len(seen) rounded to bf16 as a probability
            assert set(np.nonzero(got[n, h])[0]) == seen               # exactly the visible keys


def test_kv_write_read_roundtrip_and_compact_bit_exact():
    cfg = bf16_shape()
    W = make_weights(cfg)
    parent = frozen_tree("prior64")
    tree = O.Tree(parent)
    B, T, L = 2, tree.T, 45
    sess = gpu_session(cfg, parent, B, 128, W, page_perm_seed=9)
    m = oracle_model(cfg, W)
    rng = np.random.default_rng(4)
    caches = [O.FlatCache(m, L + T) for _ in range(B)]
    for c in caches:
        c.K[:] = cache_round(rng.standard_normal(c.K.shape)); c.V[:] = cache_round(rng.standard_normal(c.V.shape))
    load_oracle_cache(sess, caches, L + T)
    sess.seq_len.fill_(L)
    back = read_cache(sess, sess.main, 0, L + T)
    for b in range(B):
        for l in range(cfg.NL):
            np.testing.assert_array_equal(back[l, b, :, 0], caches[b].K[l]); np.testing.assert_array_equal(back[l, b, :, 1], caches[b].V[l])
    paths = [[0, 2, 9, 30, 50], [0, 1]]
    o = sess.out()
    P = tree.max_depth + 1
    o.path.copy_(torch.tensor([p + [-1] * (P - len(p)) for p in paths], dtype=torch.int32))
    o.n_acc.copy_(torch.tensor([len(p) for p in paths], dtype=torch.int32))
    o.last_node.copy_(torch.tensor([p[-1] for p in paths], dtype=torch.int32))
    o.next_root.copy_(torch.tensor([5, 6], dtype=torch.int32))
    sess.compact()
    torch.cuda.synchronize()
    after = read_cache(sess, sess.main, 0, L + T)
    for b in range(B):
        assert int(sess.seq_len[b]) == O.kv_compact(caches[b], L, paths[b])
        for l in range(cfg.NL):
            np.testing.assert_array_equal(after[l, b, :, 0], caches[b].K[l]); np.testing.assert_array_equal(after[l, b, :, 1], caches[b].V[l])


def _audit_children(logits, kids, tol_abs):
    ref = O.top_k_ids(logits, len(kids))
    if kids == ref:
        return True
    vals = logits[kids]
    assert len(set(kids)) == len(kids)
    assert np.all(np.diff(vals) <= tol_abs), "children not in descending order beyond tolerance"
    assert vals[-1] >= logits[ref[-1]] - tol_abs, "a child is not among the top-k within tolerance"
    return False


@pytest.mark.parametrize("tree_name,B,mlp", [("prior64", 1, 1), ("prior64", 2, 4), ("tiny16", 5, 2), ("prior128", 1, 1), ("single", 1, 1),
                                             ("sweep12", 2, 1), ("sweep24", 1, 4), ("sweep48", 3, 1),
                                             ("prior64", 16, 2)])                          # 336 draft rows in the widest phase
def test_draft_tree_matches_oracle(tree_name, B, mlp):
    print("case", tree_name, B, mlp, flush=True)
    cfg = bf16_shape(mlp_layers=mlp)
    W = make_weights(cfg, std=0.06)
    parent = TREES[tree_name]()
    tree = O.Tree(parent)
    m = oracle_model(cfg, W)
    sess = gpu_session(cfg, parent, B, 32, W)
    rng = np.random.default_rng(5)
    h = rng.standard_normal((B, cfg.d)).astype(np.float32)
    roots = uniform_tokens(5, 0, B, cfg.V)
    sess.h_last.copy_(torch.tensor(h)); sess.root.copy_(roots)
    sess.draft()
    torch.cuda.synchronize()
    got = sess.out().tree_tokens.cpu().tolist()
    exact = audited = 0
    for b in range(B):
        assert got[b][0] == int(roots[b])
        _, lg = O.draft_tree(m, tree, h[b].astype(np.float64), int(roots[b]), forced_tokens=got[b])
        for n, logits in lg.items():
            kids = [got[b][c] for c in tree.children[n]]
            if _audit_children(logits, kids, TOL * np.max(np.abs(logits))):
                exact += 1
            else:
                audited += 1
    print("nodes exact:", exact, "nodes with near-tie reorderings:", audited, flush=True)
    assert exact >= audited
    assert sess.main.read_flags() == 0


@pytest.mark.parametrize("tree_name,B,L", [("prior64", 1, 37), ("prior64", 2, 64), ("tiny16", 3, 5), ("single", 2, 90),
                                            ("prior128", 1, 130), ("chain40", 1, 0), ("random70", 2, 33),
                                            ("sweep12", 3, 50), ("sweep24", 2, 7), ("sweep48", 1, 100),
                                            ("prior64", 16, 21), ("prior128", 3, 9)])      # 1024 and 384 rows: several row groups per GEMM
def test_tree_verify_forward_teacher_forced(tree_name, B, L):
    _verify_forward_teacher_forced(tree_name, B, L)


@pytest.mark.parametrize("min_wgs", [1, 20])
def test_tree_verify_forward_many_rows_kernel_on_a_small_model(min_wgs, monkeypatch):
    """1024 rows with the planner's workgroup threshold lowered, so that every GEMM of the small model (residual and
    plain epilogues included) takes the kernel that shares the X tiles through LDS: eight waves (threshold 1) or
    four where eight would leave too few workgroups (threshold 20)."""
    monkeypatch.setenv("HYDRA_PLAN_SHARED_X_MIN_WGS", str(min_wgs))
    _verify_forward_teacher_forced("prior64", 16, 21)


@pytest.mark.parametrize("splits", [2, 3])
def test_tree_verify_forward_many_rows_kernel_with_k_split_over_workgroups(splits, monkeypatch):
    """The same kernel with K also split over workgroups wherever the output is a plain partial sum (O, down, LM head):
    two and three splits, the latter with a ragged last split in the down projection (24 k-steps in blocks of four)."""
    monkeypatch.setenv("HYDRA_PLAN_SHARED_X_MIN_WGS", "1")
    monkeypatch.setenv("HYDRA_PLAN_SHARED_X_SPLITS", str(splits))
    _verify_forward_teacher_forced("prior64", 16, 21)


@pytest.mark.parametrize("tree_name,B,L", [("prior64", 1, 21), ("tiny16", 3, 17), ("single", 2, 9), ("prior32", 1, 40)])
def test_tree_verify_forward_two_band_pairs_per_wave(tree_name, B, L, monkeypatch):
    """The q|k|v GEMM with two band pairs per wave (the planner takes that shape when one pair per wave would need a
    second, mostly empty round of workgroups, as at the 33B width); forced here on the small model, 1 and 2 row blocks."""
    monkeypatch.setenv("HYDRA_PLAN_PAIRS_NT", "4")
    _verify_forward_teacher_forced(tree_name, B, L)


@pytest.mark.parametrize("tree_name,B,L", [("prior64", 1, 21), ("tiny16", 3, 17), ("prior32", 2, 40)])
def test_tree_verify_forward_five_bands_per_wave_in_gate_up(tree_name, B, L, monkeypatch):
    """The gate/up GEMM with five bands per wave (the planner takes that shape for very wide FFNs, where four would
    need a second round of workgroups); forced here on the small model, whose 24 bands leave the last wave a ragged four."""
    monkeypatch.setenv("HYDRA_PLAN_SWIGLU_NT", "5")
    _verify_forward_teacher_forced(tree_name, B, L)


@pytest.mark.parametrize("tree_name,B,L", [("prior64", 2, 33), ("prior128", 1, 200), ("tiny16", 3, 0), ("prior64", 1, 95)])
def test_tree_verify_forward_with_rotary_and_append_as_their_own_kernel(tree_name, B, L, monkeypatch):
    """Beyond 128 rows the planner may split K of the q|k|v GEMM over workgroups and leave rotary embedding and cache
    append to a second kernel (which has to undo the pairing of the packed q and k bands); forced here for every shape."""
    monkeypatch.setenv("HYDRA_PLAN_QKV_UNFUSED", "1")
    _verify_forward_teacher_forced(tree_name, B, L)


def test_tree_verify_forward_is_bitwise_the_same_without_the_kv_pre_read(monkeypatch):
    """The spare workgroups of the q|k|v launch only read cached K/V pages ahead of attention; switching them off
    must not change a single bit of any output (rows of different lengths, one of them empty)."""
    cfg = bf16_shape()
    W = make_weights(cfg, gain_std=0.1, std=0.05)
    parent = TREES["prior64"]()
    T = len(parent)
    B, lens = 3, [150, 0, 37]
    sess = gpu_session(cfg, parent, B, 200, W, page_perm_seed=3, want_logits=True)
    rng = np.random.default_rng(8)
    for l in range(cfg.NL):
        t = torch.tensor(rng.standard_normal((B, max(lens), 2, cfg.H, cfg.Dh)) * 0.5, dtype=torch.float32, device="cuda:0")
        sess.main.kv_write(B, l, sess.kv, 0, max(lens), t)
    o = sess.out()
    toks = torch.stack([uniform_tokens(8, b, T, cfg.V) for b in range(B)]).to(torch.int32)
    outs = []
    for mode in ("1", "0"):
        monkeypatch.setenv("HYDRA_KV_TOUCH", mode)
        sess.seq_len.copy_(torch.tensor(lens, dtype=torch.int32)); sess.host_len = max(lens)
        o.tree_tokens.copy_(toks)
        sess.verify()
        torch.cuda.synchronize()
        assert sess.main.read_flags() == 0
        outs.append((o.hidden.clone(), o.logits.clone(), o.argmax.clone(), o.margin.clone()))
    for a, b in zip(*outs):
        assert torch.equal(a, b)


@pytest.mark.parametrize("tree_name,B", [("prior64", 1), ("tiny16", 3), ("prior128", 1), ("single", 2)])
def test_greedy_token_and_margin_without_a_logits_buffer(tree_name, B, monkeypatch):
    """Without a logits buffer the LM head's epilogue keeps two candidates per 32-column band and a small kernel merges
    them; with one, the logits go through memory.  Same inputs through both: hidden states bit-equal, margins
    bit-equal, tokens equal (a token may differ only where the margin is exactly 0: a tie after scaling).  The
    vocabulary (1000) ends inside a band.  The band-wise path is opt-in (HYDRA_LM_HEAD_TOP2=1); without the switch a
    call without a logits buffer must give the same bits too."""
    cfg = bf16_shape()
    W = make_weights(cfg, gain_std=0.1, std=0.05)
    parent = TREES[tree_name]()
    T = len(parent)
    lens = [90, 0, 37][:B]
    rng = np.random.default_rng(21)
    kvs = [torch.tensor(rng.standard_normal((B, max(lens) + 1, 2, cfg.H, cfg.Dh)) * 0.5, dtype=torch.float32, device="cuda:0") for _ in range(cfg.NL)]
    toks = torch.stack([uniform_tokens(21, b, T, cfg.V) for b in range(B)]).to(torch.int32)
    outs = {}
    for mode, want, env in (("logits", True, "1"), ("top2", False, "1"), ("top2-off", False, "0")):
        monkeypatch.setenv("HYDRA_LM_HEAD_TOP2", env)
        sess = gpu_session(cfg, parent, B, 160, W, page_perm_seed=3, want_logits=want)
        for l in range(cfg.NL):
            sess.main.kv_write(B, l, sess.kv, 0, max(lens) + 1, kvs[l])
        sess.seq_len.copy_(torch.tensor(lens, dtype=torch.int32)); sess.host_len = max(lens)
        o = sess.out()
        o.tree_tokens.copy_(toks)
        sess.verify()
        torch.cuda.synchronize()
        assert sess.main.read_flags() == 0
        outs[mode] = (o.hidden.clone(), o.argmax.clone(), o.margin.clone(), o.logits.clone() if want else None)
    h0, a0, m0, lg = outs["logits"]
    # the logits path is self-consistent (lowest-index maximum, top-1 minus top-2)
    top2 = torch.topk(lg, 2, dim=-1).values
    assert torch.equal(m0, top2[..., 0] - top2[..., 1])
    for mode in ("top2", "top2-off"):
        h, a, m, _ = outs[mode]
        assert torch.equal(h, h0) and torch.equal(m, m0), mode
        differ = a != a0
        assert not bool((differ & (m0 != 0)).any()), mode
        picked = torch.gather(lg, 2, a.long().unsqueeze(-1)).squeeze(-1)
        assert torch.equal(picked, top2[..., 0]), mode           # whatever was picked carries the maximal logit
    print(tree_name, B, "tokens that differ at an exact tie:", int((outs["top2"][1] != a0).sum()), flush=True)


def _verify_forward_teacher_forced(tree_name, B, L):
    print("case", tree_name, B, L, flush=True)
    cfg = bf16_shape()
    W = make_weights(cfg, gain_std=0.1, std=0.05)
    parent = TREES[tree_name]()
    tree = O.Tree(parent)
    T = tree.T
    m = oracle_model(cfg, W)
    sess = gpu_session(cfg, parent, B, L + 32, W, page_perm_seed=2, want_logits=True)
    caches, toks = [], []
    for b in range(B):
        c = O.FlatCache(m, L + T)
        if L:
            O.ar_prefill(m, c, uniform_tokens(6, b, L, cfg.V).tolist())
        caches.append(c)
        toks.append(uniform_tokens(6, 100 + b, T, cfg.V).tolist())
    load_oracle_cache(sess, caches, L)
    sess.seq_len.fill_(L)
    o = sess.out()
    o.tree_tokens.copy_(torch.tensor(toks, dtype=torch.int32))
    sess.verify()
    torch.cuda.synchronize()
    assert sess.main.read_flags() == 0
    newkv = read_cache(sess, sess.main, L, T)
    audit = VerifyAudit(TOL)
    worst_h = 0.0
    for b in range(B):
        hid, logits, amax = O.tree_verify(m, caches[b], L, tree, toks[b])
        worst_h = max(worst_h, max_rel(to_np(o.hidden[b]), hid))
        audit.add(o.logits[b].cpu().numpy(), o.argmax[b].cpu().numpy(), o.margin[b].cpu().numpy(), logits, amax)
        for l in range(cfg.NL):
            assert max_rel(newkv[l, b, :, 0].reshape(T, -1), caches[b].K[l, L:L + T].reshape(T, -1)) <= TOL
            assert max_rel(newkv[l, b, :, 1].reshape(T, -1), caches[b].V[l, L:L + T].reshape(T, -1)) <= TOL
    print("hidden err", worst_h, flush=True)
    assert worst_h <= TOL
    audit.finish(f"{tree_name} B={B} L={L}", max_skip_frac=0.3)


def test_generation_free_running_until_first_near_tie():
    """Prefill + Hydra steps on the GPU, free running, against oracle greedy decoding."""
    cfg = bf16_shape(K=4)
    W = make_weights(cfg, gain_std=0.1, std=0.05)
    m = oracle_model(cfg, W)
    parent = frozen_tree("prior64")
    prompt = uniform_tokens(77, 0, 70, cfg.V)
    n_new = 12
    truth = O.ar_generate(m, prompt.tolist(), n_new)
    sess = gpu_session(cfg, parent, 1, 70 + n_new + 8, W, prefill_chunk=32)
    sess.prefill(prompt.reshape(1, -1))
    toks, accs = sess.generate(n_new)
    assert sess.main.read_flags() == 0
    agree = next((j for j in range(n_new) if toks[0][j] != truth[j]), n_new)
    print("tokens agreeing before the first difference:", agree, "of", n_new, flush=True)
    if agree < n_new:
        cache = O.FlatCache(m, len(prompt) + agree + 1)
        _, _, _, lg = O.ar_prefill(m, cache, prompt.tolist() + truth[:agree])
        assert near_tie(lg, TOL), "first differing token is not a near-tie of the oracle"
