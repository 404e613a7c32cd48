"""Stored expected values (tests/golden/, written by tests/golden/make_golden.py from the oracle alone).

CPU: the oracle still reproduces the stored tokens, and Hydra decoding's stored tokens equal plain
greedy decoding's (greedy acceptance does not change the output: paper section 5 "Evaluation").
GPU: the library's free-running generation equals the stored tokens.
"""
import json
import os

import pytest

from oracle import hydra_oracle as O
from synth import CONFIGS, frozen_tree, uniform_tokens
from helpers import make_weights, oracle_model

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "config1_greedy.json")))


def test_stored_hydra_tokens_equal_stored_greedy_tokens():
    assert GOLD["hydra_tokens"] == GOLD["greedy_tokens"]
    assert sum(GOLD["hydra_acceptance"]) >= len(GOLD["greedy_tokens"])
    assert all(1 <= a <= 4 for a in GOLD["hydra_acceptance"])
    assert len(GOLD["first_draft_tree_tokens"]) == 16


def test_oracle_reproduces_stored_tokens():
    cfg = CONFIGS[1]
    assert cfg.seed == GOLD["seed"]
    m = oracle_model(cfg, make_weights(cfg, gain_std=0.0))
    prompt = uniform_tokens(cfg.seed, 0, cfg.prompt[0], cfg.V).tolist()
    assert prompt[:8] == GOLD["prompt_head"]
    assert O.ar_generate(m, prompt, 24) == GOLD["greedy_tokens"][:24]
    toks, acc = O.hydra_generate(m, O.Tree(frozen_tree("tiny16")), prompt, 24)
    assert toks == GOLD["greedy_tokens"][:24]
    assert acc == GOLD["hydra_acceptance"][:len(acc)]


@pytest.mark.gpu
def test_library_generation_equals_stored_tokens():
    import torch
    from gpu_util import generate_checked, gpu_session
    cfg = CONFIGS[1]
    W = make_weights(cfg, gain_std=0.0)
    prompt = uniform_tokens(cfg.seed, 0, cfg.prompt[0], cfg.V)
    make = lambda: gpu_session(cfg, frozen_tree("tiny16"), 1, cfg.prompt[0] + cfg.gen + 8, W, prefill_chunk=32)
    sess = make()
    sess.prefill(prompt.reshape(1, -1))
    sess.draft()
    torch.cuda.synchronize()
    first_tree = sess.out().tree_tokens[0].cpu().tolist()
    truth = GOLD["greedy_tokens"]
    segments, near_ties = generate_checked(make, prompt, truth, cfg.gen, oracle_model(cfg, W), 1e-4)
    accs = segments[0][2]
    if near_ties:                                         # acceptance lengths are comparable up to the first restart
        emitted, keep = 0, 0
        for a in accs:
            if emitted + a[0] > len(segments[0][1]):
                break
            emitted += a[0]; keep += 1
        accs = accs[:keep]
    assert [a[0] for a in accs] == GOLD["hydra_acceptance"][:len(accs)]
    assert first_tree == GOLD["first_draft_tree_tokens"]
