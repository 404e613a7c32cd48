"""Seeded random-init weights for a Llama-shape decoder plus Hydra draft heads.

Every matrix and MLP bias is i.i.d. ~N(0, 0.02^2); RMSNorm gains are 1 (or
1 + N(0, gain_std^2) when a test wants gains that matter).  Tensors are made one
at a time, by name, so a caller can stream a 33B-shape model through a device
without ever holding a second copy.

Tensor names and shapes (row-major, [out_features, in_features]):
    embed [V,d]  lm_head [V,d]  final_norm [d]
    layers.L.attn_norm [d]  layers.L.wq|wk|wv|wo [d,d]
    layers.L.ffn_norm [d]   layers.L.w_gate|w_up [F,d]  layers.L.w_down [d,F]
    heads.I.w1 [d,(I+1)d]  (or [d, I*d] without the root embedding; [d, d] for Medusa-style heads), heads.I.b1 [d]
    heads.I.wJ [d,d], heads.I.bJ [d]  for J = 2..mlp_layers
    heads.I.wout [V,d]                                   I = 1..K
    prefix.<same nine names as a decoder layer>          when the configuration has the prefix-attention layer
"""
from __future__ import annotations

from dataclasses import dataclass

import torch

from .configs import ModelShape
from .rng import normal_tensor


@dataclass(frozen=True)
class WeightSpec:
    shape_cfg: ModelShape
    std: float = 0.02
    gain_std: float = 0.0

    def head_in_width(self, i: int) -> int:
        c = self.shape_cfg
        if c.medusa:
            return c.d
        return (i + 1) * c.d if c.include_root_embedding else i * c.d


def tensor_names(cfg: ModelShape) -> list:
    names = ["embed", "lm_head", "final_norm"]
    for l in range(cfg.NL):
        for t in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down"):
            names.append(f"layers.{l}.{t}")
    for i in range(1, cfg.K + 1):
        names += [f"heads.{i}.w1", f"heads.{i}.b1"]
        for j in range(2, cfg.mlp_layers + 1):
            names += [f"heads.{i}.w{j}", f"heads.{i}.b{j}"]
        names.append(f"heads.{i}.wout")
    if cfg.prefix:
        names += [f"prefix.{t}" for t in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")]
    return names


_LAYER_SLOT = {"attn_norm": 0, "wq": 1, "wk": 2, "wv": 3, "wo": 4, "ffn_norm": 5,
               "w_gate": 6, "w_up": 7, "w_down": 8}


def _tensor_id_and_shape(spec: WeightSpec, name: str):
    c = spec.shape_cfg
    parts = name.split(".")
    if name == "embed":
        return 1, (c.V, c.d), "matrix"
    if name == "lm_head":
        return 2, (c.V, c.d), "matrix"
    if name == "final_norm":
        return 3, (c.d,), "gain"
    if parts[0] in ("layers", "prefix"):
        if parts[0] == "layers":
            l, t = int(parts[1]), parts[2]
            tid = 1000 + l * 16 + _LAYER_SLOT[t]
        else:
            t = parts[1]
            tid = 500 + _LAYER_SLOT[t]
        if t in ("attn_norm", "ffn_norm"):
            return tid, (c.d,), "gain"
        if t in ("wq", "wk", "wv", "wo"):
            return tid, (c.d, c.d), "matrix"
        if t in ("w_gate", "w_up"):
            return tid, (c.F, c.d), "matrix"
        if t == "w_down":
            return tid, (c.d, c.F), "matrix"
    if parts[0] == "heads":
        i, t = int(parts[1]), parts[2]
        base = 100000 + i * 64
        if t == "w1":
            return base, (c.d, spec.head_in_width(i)), "matrix"
        if t == "b1":
            return base + 1, (c.d,), "bias"
        if t == "wout":
            return base + 2, (c.V, c.d), "matrix"
        j = int(t[1:])
        if t[0] == "w":
            return base + 2 * j + 2, (c.d, c.d), "matrix"
        if t[0] == "b":
            return base + 2 * j + 3, (c.d,), "bias"
    raise KeyError(name)


def tensor_shape(spec: WeightSpec, name: str) -> tuple:
    return _tensor_id_and_shape(spec, name)[1]


def make_tensor(spec: WeightSpec, name: str, device="cpu") -> torch.Tensor:
    """The named tensor in the configuration's storage dtype (fp32 or bf16)."""
    c = spec.shape_cfg
    tid, shape, kind = _tensor_id_and_shape(spec, name)
    dtype = torch.bfloat16 if c.dtype == "bf16" else torch.float32
    if kind == "gain":
        if spec.gain_std == 0.0:
            return torch.ones(shape, dtype=dtype, device=device)
        g = normal_tensor(c.seed, tid, shape, std=spec.gain_std, dtype=torch.float32, device=device)
        return (g + 1.0).to(dtype)
    return normal_tensor(c.seed, tid, shape, std=spec.std, dtype=dtype, device=device)
