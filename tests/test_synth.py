"""The seeded input generators: determinism, distribution, frozen trees."""
import collections
import json
import os

import torch

from synth import (CONFIGS, WeightSpec, build_prior_tree, chain_tree, frozen_tree, make_tensor,
                   normal_tensor, random_tree, tensor_names, uniform_tokens)
from synth.trees import paths_from_parent, tree_from_paths, _regenerate_frozen
from synth.weights import tensor_shape


def test_normal_tensor_is_deterministic_and_chunk_independent():
    a = normal_tensor(5, 9, (1000, 37))
    b = normal_tensor(5, 9, (1000, 37), chunk=4099)
    assert torch.equal(a, b)
    assert not torch.equal(a, normal_tensor(5, 10, (1000, 37)))
    assert not torch.equal(a, normal_tensor(6, 9, (1000, 37)))


def test_normal_tensor_moments():
    x = normal_tensor(1, 1, (1 << 20,), std=0.02).double()
    assert abs(x.mean().item()) < 1e-4
    assert abs(x.std().item() / 0.02 - 1) < 5e-3
    k = ((x / 0.02) ** 4).mean().item()
    assert abs(k - 2.9) < 0.05                      # Irwin-Hall(12): kurtosis 3 - 0.1
    assert x.abs().max().item() <= 6 * 0.02


def test_bf16_tensor_is_rounding_of_fp32_tensor():
    a = normal_tensor(2, 3, (257, 33), dtype=torch.float32)
    b = normal_tensor(2, 3, (257, 33), dtype=torch.bfloat16)
    assert torch.equal(a.to(torch.bfloat16), b)


def test_uniform_tokens_in_range_and_spread():
    t = uniform_tokens(3, 0, 100000, 1024)
    assert t.dtype == torch.int32 and int(t.min()) >= 0 and int(t.max()) < 1024
    counts = torch.bincount(t.long(), minlength=1024)
    assert int(counts.min()) > 50 and int(counts.max()) < 160
    assert not torch.equal(t[:100], uniform_tokens(3, 1, 100, 1024))


def test_every_tensor_name_has_the_documented_shape():
    cfg = CONFIGS[1]
    spec = WeightSpec(cfg)
    names = tensor_names(cfg)
    assert len(names) == 3 + 9 * cfg.NL + cfg.K * 3
    for i in range(1, cfg.K + 1):
        assert tensor_shape(spec, f"heads.{i}.w1") == (cfg.d, (i + 1) * cfg.d)   # input width grows with i
    ids = set()
    from synth.weights import _tensor_id_and_shape
    for n in names:
        tid, shape, _ = _tensor_id_and_shape(spec, n)
        assert tid not in ids
        ids.add(tid)
        assert tuple(make_tensor(spec, n).shape) == shape if len(shape) == 1 or shape[0] * shape[1] < 1 << 20 else True
    spec4 = WeightSpec(CONFIGS[3])
    assert tensor_shape(spec4, "heads.2.w4") == (4096, 4096)


def test_frozen_trees_match_the_builder_and_the_stated_shapes():
    here = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "synth", "trees_frozen.json")
    frozen = json.load(open(here))
    assert frozen == json.loads(json.dumps(_regenerate_frozen()))
    per_depth = {"tiny16": [1, 4, 7, 4], "prior32": [1, 6, 14, 10, 1], "prior64": [1, 7, 21, 20, 15],
                 "prior128": [1, 8, 28, 56, 35]}
    expanding = {"tiny16": [1, 3, 3], "prior32": [1, 4, 6, 1], "prior64": [1, 6, 10, 10], "prior128": [1, 7, 21, 20]}
    for name, want in per_depth.items():
        parent = frozen_tree(name)
        paths = paths_from_parent(parent)
        cnt = collections.Counter(len(p) for p in paths)
        assert [cnt[d] for d in range(len(want))] == want
        exp = collections.Counter(len(paths[p]) for p in set(parent) if p >= 0)
        assert [exp[d] for d in range(len(expanding[name]))] == expanding[name]
        assert tree_from_paths(paths) == parent
        assert all(parent[n] < n for n in range(1, len(parent)))
    assert [tuple(p) for p in frozen["tiny16"]["paths"]] == [
        (), (0,), (1,), (2,), (3,), (0, 0), (0, 1), (0, 2), (1, 0), (1, 1), (1, 2), (2, 0),
        (0, 0, 0), (0, 0, 1), (0, 1, 0), (1, 0, 0)]


def test_helper_trees_are_bfs_ordered():
    for parent in (chain_tree(6), random_tree(20, 4, 1), random_tree(33, 3, 2), build_prior_tree(10, (3, 3, 3))):
        assert parent[0] == -1
        depth = [0] * len(parent)
        for n in range(1, len(parent)):
            assert 0 <= parent[n] < n
            depth[n] = depth[parent[n]] + 1
            assert depth[n] >= depth[n - 1]                 # BFS: depth never decreases
            assert parent[n] >= parent[n - 1]               # children of a node are contiguous


# ---- proposal trees of the tree-size sweep and their expected acceptance length ---------------------------------
def _brute_force_expected_acceptance(parent, caps):
    """Enumerates every outcome of the synthetic acceptance model: at depth j the base model's token is the rank-r
    candidate with probability q(j, r), or none of the ranks with the rest; the step accepts the longest prefix of
    the outcome's rank path that is a node of the tree.  Written from the model's statement, not from the sum over
    nodes that expected_acceptance uses."""
    from fractions import Fraction
    from itertools import product
    from synth import paths_from_parent
    nodes = set(paths_from_parent(parent))
    q = lambda j, r: Fraction(3, 10) * Fraction(8, 10) ** j * Fraction(1, 2) ** r
    total, mass = Fraction(0), Fraction(0)
    choices = [list(range(c)) + [None] for c in caps]
    for outcome in product(*choices):
        p = Fraction(1)
        for j, r in enumerate(outcome):
            p *= q(j, r) if r is not None else 1 - sum(q(j, rr) for rr in range(caps[j]))
        mass += p
        length, path = 1, ()
        for r in outcome:
            if r is None or path + (r,) not in nodes:
                break
            path += (r,)
            length += 1
        total += p * length
    assert mass == 1
    return total


def test_expected_acceptance_equals_enumeration_of_all_outcomes():
    from synth import expected_acceptance, proposal_trees, tree_from_paths
    caps = (3, 3, 2)
    for parent in proposal_trees(12, caps) + [tree_from_paths([(), (0,), (1,), (0, 0), (0, 1), (1, 0), (0, 0, 0), (0, 0, 1), (1, 0, 0)])]:
        assert expected_acceptance(parent) == _brute_force_expected_acceptance(parent, caps)
    assert expected_acceptance([-1]) == 1


def test_proposal_trees_are_nested_valid_and_greedy():
    from fractions import Fraction
    from synth import accept_prob, expected_acceptance, paths_from_parent, proposal_trees
    trees = proposal_trees(128)
    assert [len(t) for t in trees] == list(range(1, 129))
    prev_paths, prev_e = set(), Fraction(0)
    for t in trees:
        paths = paths_from_parent(t)
        assert paths == sorted(paths, key=lambda p: (len(p), p))              # breadth-first order
        assert all(t[n] < n for n in range(1, len(t))) and max(len(p) for p in paths) <= 4
        s = set(paths)
        assert prev_paths < s or not prev_paths                               # nested: one node more each time
        added = s - prev_paths
        if prev_paths:
            (new,) = added
            # greedy: no absent node whose parent and previous sibling are present is more probable than the one added
            for p in prev_paths:
                r = 0
                while p + (r,) in prev_paths:
                    r += 1
                if len(p) < 4 and r < 10:
                    assert accept_prob(p + (r,)) <= accept_prob(new)
        e = expected_acceptance(t)
        assert e > prev_e
        prev_paths, prev_e = s, e
    assert 1 < float(expected_acceptance(trees[63])) < 2                      # a modest prior: about 1.8 tokens per step at 64 nodes
