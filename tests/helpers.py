"""Shared test plumbing: build an oracle model from the seeded generators."""
from __future__ import annotations

import torch

from oracle import hydra_oracle as O
from synth import ModelShape, WeightSpec, make_tensor, tensor_names


def small_shape(**kw) -> ModelShape:
    base = dict(name="t", d=32, NL=2, H=4, Dh=8, F=48, V=97, dtype="f32", K=3, mlp_layers=1,
                T=8, batch=(1,), prompt=(12,), gen=8, seed=1234)
    base.update(kw)
    return ModelShape(**base)


def make_weights(cfg: ModelShape, gain_std=0.1, std=0.02, device="cpu") -> dict:
    spec = WeightSpec(cfg, std=std, gain_std=gain_std)
    return {n: make_tensor(spec, n, device=device) for n in tensor_names(cfg)}


def oracle_model(cfg: ModelShape, weights: dict, keep=True) -> O.Model:
    return O.Model(cfg.d, cfg.NL, cfg.H, cfg.Dh, cfg.F, cfg.V, cfg.K, cfg.mlp_layers, weights,
                   rms_eps=cfg.rms_eps, rope_theta=cfg.rope_theta,
                   include_root_embedding=cfg.include_root_embedding, keep_converted=keep, medusa=cfg.medusa)
