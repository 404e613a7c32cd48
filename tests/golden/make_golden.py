#!/usr/bin/env python3
"""Writes the stored expected values under tests/golden/ from the CPU oracle alone.

    python tests/golden/make_golden.py

config1_greedy.json: the tiny fp32 configuration (d = 256, 2 layers, 4 heads of 64, V = 1024,
3 Hydra heads, 16-node tree), 128-token seeded prompt, 64 tokens of plain greedy decoding by the
float64 oracle, the tokens and acceptance lengths of Hydra decoding with greedy acceptance over
the same prompt (which must be the same tokens: greedy acceptance leaves the output unchanged,
paper section 5 "Evaluation"), and the first step's draft tree.  Nothing here calls the GPU library.
"""
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
sys.path.insert(0, os.path.dirname(HERE))

from oracle import hydra_oracle as O                                    # noqa: E402
from synth import CONFIGS, frozen_tree, uniform_tokens                  # noqa: E402
from helpers import make_weights, oracle_model                          # noqa: E402


def main():
    cfg = CONFIGS[1]
    W = make_weights(cfg, gain_std=0.0)
    m = oracle_model(cfg, W)
    prompt = uniform_tokens(cfg.seed, 0, cfg.prompt[0], cfg.V).tolist()
    tree = O.Tree(frozen_tree("tiny16"))
    greedy = O.ar_generate(m, prompt, cfg.gen)
    hydra, acc = O.hydra_generate(m, tree, prompt, cfg.gen)
    cache = O.FlatCache(m, len(prompt) + tree.T + 4)
    L, h_last, root, _ = O.ar_prefill(m, cache, prompt)
    tok, _ = O.draft_tree(m, tree, h_last, root)
    out = {"source": "oracle/hydra_oracle.py via tests/golden/make_golden.py", "config": 1, "seed": cfg.seed,
           "prompt_len": len(prompt), "prompt_head": prompt[:8], "tree": "tiny16",
           "greedy_tokens": [int(t) for t in greedy], "hydra_tokens": [int(t) for t in hydra],
           "hydra_acceptance": [int(a) for a in acc], "first_draft_tree_tokens": [int(t) for t in tok]}
    with open(os.path.join(HERE, "config1_greedy.json"), "w") as f:
        json.dump(out, f, indent=1)
        f.write("\n")
    print(out)


if __name__ == "__main__":
    main()
