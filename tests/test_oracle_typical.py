"""Pins for the oracle's typical-acceptance criterion (paper, section 6.3):
a candidate passes if p_base(token; tau) > min(eps, alpha * exp(-H(p_base(.; tau)))).

Closed forms, library routines (scipy softmax / entropy), the greedy limit, brute force over all
paths, and the distribution of the sampled next token.
"""
import itertools

import numpy as np
import pytest
from scipy.special import softmax as sp_softmax
from scipy.stats import entropy as sp_entropy

from oracle import hydra_oracle as O
from synth import frozen_tree, random_tree, star_tree


def test_uniform_distribution_closed_form():
    """All logits equal: p = 1/V for every token and H = ln V, so the threshold is min(eps, alpha / V):
    a token passes iff 1/V > min(eps, alpha/V), i.e. iff alpha < 1 or eps < 1/V."""
    V = 50
    row = np.full(V, 3.25)
    assert O.typical_pass(row, 7, tau=0.7, eps=0.3, alpha=0.9)          # alpha/V < 1/V
    assert not O.typical_pass(row, 7, tau=0.7, eps=0.3, alpha=1.1)      # min(0.3, 1.1/50) = 0.022 > 0.02
    assert O.typical_pass(row, 7, tau=0.7, eps=0.01, alpha=1.1)         # eps = 0.01 < 0.02
    assert abs(O.entropy(O.tempered_probs(row, 0.7)) - np.log(V)) < 1e-12


def test_two_point_distribution_closed_form_with_temperature():
    """Two finite logits a > b, the rest -inf: p_a = 1 / (1 + exp(-(a-b)/tau)), H = -(p ln p + q ln q)."""
    a, b, tau = 1.3, 0.2, 0.7
    row = np.full(9, -np.inf); row[4], row[6] = a, b
    pa = 1.0 / (1.0 + np.exp(-(a - b) / tau)); pb = 1.0 - pa
    H = -(pa * np.log(pa) + pb * np.log(pb))
    p = O.tempered_probs(row, tau)
    assert abs(p[4] - pa) < 1e-15 and abs(p[6] - pb) < 1e-15 and p[0] == 0.0
    assert abs(O.entropy(p) - H) < 1e-15
    th = 0.5 * np.exp(-H)
    for eps in (0.05, 0.9):
        assert O.typical_pass(row, 6, tau, eps, 0.5) == (pb > min(eps, th))
        assert O.typical_pass(row, 4, tau, eps, 0.5) == (pa > min(eps, th))
    assert not O.typical_pass(row, 0, tau, 0.05, 0.5)                   # probability zero never passes


def test_against_scipy_softmax_and_entropy_and_min_not_max():
    rng = np.random.default_rng(0)
    seen_between = 0
    for _ in range(200):
        V = int(rng.integers(3, 40))
        row = rng.standard_normal(V) * 3
        tau, eps = float(rng.uniform(0.3, 1.5)), float(rng.uniform(0.02, 0.4))
        alpha = np.sqrt(eps)                                             # the paper's setting
        p = sp_softmax(row / tau)
        th_min = min(eps, alpha * np.exp(-sp_entropy(p)))
        th_max = max(eps, alpha * np.exp(-sp_entropy(p)))
        for t in range(V):
            assert O.typical_pass(row, t, tau, eps, alpha) == (p[t] > th_min)
            if th_min < p[t] <= th_max:
                seen_between += 1                                        # would be rejected under max(): the test tells them apart
    assert seen_between > 20


def test_small_temperature_reduces_to_greedy_acceptance():
    """tau -> 0: p_base(.; tau) is one-hot at the most likely token, H -> 0, the threshold is min(eps, alpha) < 1:
    exactly the greedy token passes, so typical acceptance walks the same path as greedy acceptance."""
    rng = np.random.default_rng(5)
    for trial in range(40):
        parent = random_tree(int(rng.integers(2, 20)), 3, trial)
        tree = O.Tree(parent)
        V = 11
        logits = rng.standard_normal((tree.T, V))
        amax = [O.argmax_lowest(logits[n]) for n in range(tree.T)]
        tok = rng.integers(0, V, size=tree.T)
        for n in range(tree.T):                                          # plant matches so that paths are accepted
            if tree.children[n] and rng.random() < 0.7:
                tok[tree.children[n][int(rng.integers(len(tree.children[n])))]] = amax[n]
        g = O.accept_greedy(tree, tok, amax)
        t = O.accept_typical(tree, tok, logits, tau=1e-3, eps=0.3, alpha=0.5, u=None)
        assert t[1] == g[1] or len(t[1]) == len(g[1])                    # duplicate siblings may give another equally long path
        assert t[0] == g[0] and t[2] == amax[t[3]]


def test_longest_accepted_path_equals_brute_force():
    rng = np.random.default_rng(9)
    for trial in range(60):
        parent = random_tree(int(rng.integers(1, 16)), 3, 100 + trial) if trial % 3 else star_tree(int(rng.integers(1, 9)))
        tree = O.Tree(parent)
        V = 7
        logits = rng.standard_normal((tree.T, V)) * 2
        tok = rng.integers(0, V, size=tree.T)
        tau, eps, alpha = 0.7, 0.15, np.sqrt(0.15)
        n_acc, path, nxt, last = O.accept_typical(tree, tok, logits, tau, eps, alpha)
        best = None
        for n in range(tree.T):                                          # every node ends one candidate prefix
            p = tree.path(n)
            if all(O.typical_pass(logits[tree.parent[c]], tok[c], tau, eps, alpha) for c in p[1:]):
                if best is None or len(p) > len(best):
                    best = p                                             # ascending n: the lowest id of each length is kept
        assert path == best and n_acc == len(best) and last == best[-1]
        assert nxt == O.argmax_lowest(logits[last])


def test_sampled_next_token_inverts_the_cumulative_distribution():
    p = np.array([0.0, 0.1, 0.0, 0.6, 0.3])
    assert O.sample_inverse_cdf(p, 0.0) == 1 and O.sample_inverse_cdf(p, 0.0999) == 1
    assert O.sample_inverse_cdf(p, 0.1) == 3 and O.sample_inverse_cdf(p, 0.6999) == 3
    assert O.sample_inverse_cdf(p, 0.7) == 4 and O.sample_inverse_cdf(p, 0.999999) == 4
    rng = np.random.default_rng(1)
    q = rng.random(13); q /= q.sum()
    us = (np.arange(20000) + 0.5) / 20000
    ids = np.array([O.sample_inverse_cdf(q, u) for u in us])
    assert np.all(np.diff(ids) >= 0)                                     # monotone in u
    freq = np.bincount(ids, minlength=13) / len(us)
    assert np.max(np.abs(freq - q)) < 1e-4                               # a uniform grid of u reproduces p to 1 / grid size


def test_accept_typical_uses_the_tempered_distribution_of_the_last_node():
    tree = O.Tree([-1, 0, 0])
    logits = np.array([[0.0, 5.0, 0.0, 0.0], [0.0, 0.0, 2.0, 2.0], [9.0, 0.0, 0.0, 0.0]])
    tok = [3, 1, 0]
    n_acc, path, nxt, last = O.accept_typical(tree, tok, logits, tau=0.5, eps=0.2, alpha=0.4, u=0.49)
    assert path == [0, 1] and last == 1
    p = sp_softmax(logits[1] / 0.5)
    assert nxt == int(np.searchsorted(np.cumsum(p), 0.49, side="right")) == 2
    assert O.accept_typical(tree, tok, logits, 0.5, 0.2, 0.4, u=0.51)[2] == 3


# ---- typical acceptance as a decoding loop (section 6.3 as the verification criterion of the whole procedure) ----
def _tiny_model(std=0.3, **kw):
    from helpers import make_weights, oracle_model, small_shape
    cfg = small_shape(**kw)
    return cfg, oracle_model(cfg, make_weights(cfg, gain_std=0.2, std=std))


def test_loop_with_small_temperature_reproduces_greedy_text():
    """tau -> 0 makes p one-hot on the base model's most likely token: a candidate passes iff it is that token, and the
    next root is that token, so the loop is Hydra decoding with greedy acceptance and its text is plain greedy text."""
    from synth import uniform_tokens
    cfg, m = _tiny_model()
    tree = O.Tree(frozen_tree("tiny16"))
    prompt = uniform_tokens(5, 0, 9, cfg.V).tolist()
    truth = O.ar_generate(m, prompt, 14)
    want, want_acc = O.hydra_generate(m, tree, prompt, 14)
    got, acc = O.hydra_generate(m, tree, prompt, 14, typical=(1e-3, 0.3, 0.5))
    assert got == truth == want and acc == want_acc


def test_loop_emits_only_root_paths_whose_every_token_passes_and_no_deeper_one_exists():
    """Every step of the loop: the emitted tokens are the tokens of a root path of the tree, each non-root token of it
    passes the per-token test against its parent's logits, no complete passing path is deeper (brute force over all
    root paths), the next root is the inverse of the cumulative distribution at the last node, and the next step's
    root is that token.  A flat temperature makes many candidates pass, so paths of several lengths occur."""
    from synth import uniform_tokens
    cfg, m = _tiny_model()
    tree = O.Tree(frozen_tree("tiny16"))
    prompt = uniform_tokens(6, 0, 8, cfg.V).tolist()
    tau, eps, alpha = 2.0, 0.5, 0.8
    rng = np.random.default_rng(3)
    us = rng.random(40)
    log = []
    out, acc = O.hydra_generate(m, tree, prompt, 24, typical=(tau, eps, alpha), u_per_step=us, step_log=log)
    assert len(set(acc)) >= 3 and max(acc) >= 3
    emitted = []
    for s, info in enumerate(log):
        tok, lg, path = info["tok"], info["logits"], info["path"]
        assert path[0] == 0 and all(tree.parent[path[j]] == path[j - 1] for j in range(1, len(path)))
        for j in range(1, len(path)):
            assert O.typical_pass(lg[path[j - 1]], tok[path[j]], tau, eps, alpha)
        deepest = 1
        for n in range(tree.T):                                            # brute force over all root paths
            pth = tree.path(n)
            if all(O.typical_pass(lg[pth[j - 1]], tok[pth[j]], tau, eps, alpha) for j in range(1, len(pth))):
                deepest = max(deepest, len(pth))
        assert len(path) == deepest == acc[s]
        p = O.tempered_probs(lg[path[-1]], tau)
        c = np.cumsum(p)
        v = info["next_root"]
        assert c[v] > us[s] * c[-1] and (v == 0 or c[v - 1] <= us[s] * c[-1])
        if s + 1 < len(log):
            assert log[s + 1]["tok"][0] == v                                 # the drawn token is the next step's root
        emitted += [int(tok[n]) for n in path]
    assert emitted[:24] == out
    # the same draws give the same text; other draws another one
    again, _ = O.hydra_generate(m, tree, prompt, 24, typical=(tau, eps, alpha), u_per_step=us)
    other, _ = O.hydra_generate(m, tree, prompt, 24, typical=(tau, eps, alpha), u_per_step=rng.random(40))
    assert again == out and other != out
