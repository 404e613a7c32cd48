"""Seeded synthetic inputs (weights, prompts, candidate trees, configs).

This package is the only code that both the CPU oracle's tests and the HIP
path's harness import.  It holds no arithmetic of the decoding method itself:
it only produces the numbers and tree shapes that the method is run on.
"""
from .configs import CONFIGS, ModelShape, get_config          # noqa: F401
from .rng import uniform_tokens, normal_tensor                # noqa: F401
from .trees import (build_prior_tree, chain_tree, star_tree, random_tree,      # noqa: F401
                    frozen_tree, tree_from_paths, paths_from_parent, proposal_trees, expected_acceptance, accept_prob)
from .weights import WeightSpec, tensor_names, make_tensor    # noqa: F401
