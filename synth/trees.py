"""Static candidate-tree topologies.

A tree is stored as a `parent` list in BFS order (depth, then path
lexicographic): parent[0] = -1, parent[n] < n, the children of a node are
contiguous and ordered by child rank (rank 0 = the draft's most likely token).

`build_prior_tree` grows a tree node by node, each time adding the absent child
that is worth most under a fixed synthetic acceptance prior, which is the greedy
construction of the paper's tree-discovery section with the corpus statistics
replaced by a closed-form prior (there is no corpus here):
    worth(r_1..r_k) = prod_j  0.6 * 0.8^(j-1) * 0.5^(r_j)
evaluated in exact rational arithmetic so that no float tie can change a tree.
The trees used by the workloads are frozen in `trees_frozen.json`.
"""
from __future__ import annotations

import json
import os
from fractions import Fraction

from .rng import uniform_ints

_HERE = os.path.dirname(os.path.abspath(__file__))


def tree_from_paths(paths) -> list:
    """Parent list (BFS order) from a set of child-rank paths; () is the root."""
    ps = sorted({tuple(p) for p in paths}, key=lambda p: (len(p), p))
    assert ps and ps[0] == (), "the root path () must be present"
    index = {p: i for i, p in enumerate(ps)}
    parent = []
    for p in ps:
        if not p:
            parent.append(-1)
            continue
        assert p[:-1] in index, f"path {p} has no parent in the set"
        if p[-1] > 0:
            assert p[:-1] + (p[-1] - 1,) in index, f"path {p} skips a sibling rank"
        parent.append(index[p[:-1]])
    return parent


def paths_from_parent(parent) -> list:
    """Inverse of tree_from_paths for a BFS-ordered parent list."""
    paths, next_rank = [()], {}
    for n in range(1, len(parent)):
        p = parent[n]
        r = next_rank.get(p, 0)
        next_rank[p] = r + 1
        paths.append(paths[p] + (r,))
    return paths


def _worth(path) -> Fraction:
    w = Fraction(1)
    for j, r in enumerate(path):
        w *= Fraction(6, 10) * Fraction(8, 10) ** j * Fraction(1, 2) ** r
    return w


def build_prior_tree(T: int, rank_caps) -> list:
    """Greedy growth to T nodes; rank_caps[j] = number of child ranks allowed at depth j+1."""
    have = {()}
    while len(have) < T:
        best = None
        for p in have:
            if len(p) >= len(rank_caps):
                continue
            r = 0
            while p + (r,) in have:
                r += 1
            if r >= rank_caps[len(p)]:
                continue
            cand = p + (r,)
            key = (-_worth(cand), len(cand), cand)
            if best is None or key < best[0]:
                best = (key, cand)
        if best is None:
            raise ValueError("rank caps too small for the requested tree size")
        have.add(best[1])
    return tree_from_paths(have)


# ---- proposal trees of every size and their expected acceptance length (tree-size sweep) ----------------
# The tree-discovery section of the paper grows a sequence of proposal trees T_1, T_2, ..., each by adding the node
# with the highest expected contribution to the acceptance length, estimated on a corpus, and then measures which
# size gives the highest throughput.  There is no corpus here; the sweep uses a synthetic acceptance model that is a
# proper probability model, so that "expected acceptance length" has a meaning:
#   given that the path above it is accepted, the rank-r candidate of the head at depth j is the base model's next
#   token with probability  q(j, r) = 0.3 * 0.8^(j-1) * 0.5^r        (sum over r below 1 at every depth).
# Siblings are distinct tokens, so at most one child of a node is accepted, and
#   P(node accepted) = product of q over the edges of its root path,
#   E[acceptance length] = sum over all nodes of P(node accepted)   (the root counts 1).
# Greedy growth by P(node accepted) therefore yields, for every size, a tree of maximal expected acceptance length,
# and the trees are nested.  Numbers derived from it are properties of this synthetic prior, not corpus statistics.

def accept_prob(path) -> Fraction:
    """P(the node with this child-rank path lies on the accepted path) under the synthetic acceptance model."""
    w = Fraction(1)
    for j, r in enumerate(path):
        w *= Fraction(3, 10) * Fraction(8, 10) ** j * Fraction(1, 2) ** r
    return w


def expected_acceptance(parent) -> Fraction:
    """Expected number of tokens a step accepts with this tree under the synthetic acceptance model (root included)."""
    return sum((accept_prob(p) for p in paths_from_parent(parent)), Fraction(0))


def proposal_trees(N: int, rank_caps=(10, 10, 10, 10)) -> list:
    """[T_1, ..., T_N] as parent lists: T_n has n nodes and adds to T_{n-1} the absent node of highest acceptance
    probability whose parent and previous sibling are present (ties: shallower, then lexicographic)."""
    have = {()}
    out = [tree_from_paths(have)]
    while len(have) < N:
        best = None
        for p in have:
            if len(p) >= len(rank_caps):
                continue
            r = 0
            while p + (r,) in have:
                r += 1
            if r >= rank_caps[len(p)]:
                continue
            cand = p + (r,)
            key = (-accept_prob(cand), len(cand), cand)
            if best is None or key < best[0]:
                best = (key, cand)
        if best is None:
            raise ValueError("rank caps too small for the requested tree size")
        have.add(best[1])
        out.append(tree_from_paths(have))
    return out


def chain_tree(T: int) -> list:
    return [-1] + list(range(T - 1))


def star_tree(m: int) -> list:
    return [-1] + [0] * m


def random_tree(T: int, max_depth: int, seed: int) -> list:
    """Uniformly random attachment under a depth cap, returned in BFS order."""
    draws = uniform_ints(seed, T, 4 * T + 8, 1 << 30)
    parent, depth, it = [-1], [0], 0
    while len(parent) < T:
        cand = draws[it % len(draws)] % len(parent)
        it += 1
        if depth[cand] < max_depth:
            parent.append(cand)
            depth.append(depth[cand] + 1)
        elif it > 64 * T:
            raise ValueError("could not place all nodes under the depth cap")
    # convert to rank paths, then to BFS order
    paths, nrank = [()], {}
    for n in range(1, T):
        p = parent[n]
        r = nrank.get(p, 0)
        nrank[p] = r + 1
        paths.append(paths[p] + (r,))
    return tree_from_paths(paths)


def frozen_tree(name: str) -> list:
    """One of the frozen workload trees: 'tiny16', 'prior32', 'prior64', 'prior128'."""
    with open(os.path.join(_HERE, "trees_frozen.json")) as f:
        return json.load(f)[name]["parent"]


def _regenerate_frozen() -> dict:
    out = {}
    for name, T, caps in (("tiny16", 16, (4, 3, 2)), ("prior32", 32, (10, 10, 10, 10)),
                          ("prior64", 64, (10, 10, 10, 10)), ("prior128", 128, (10, 10, 10, 10))):
        parent = build_prior_tree(T, caps)
        out[name] = {"T": T, "rank_caps": list(caps), "parent": parent,
                     "paths": [list(p) for p in paths_from_parent(parent)]}
    return out


if __name__ == "__main__":
    with open(os.path.join(_HERE, "trees_frozen.json"), "w") as f:
        json.dump(_regenerate_frozen(), f, indent=1)
