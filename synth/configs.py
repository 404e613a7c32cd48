"""The five workload configurations of this build, as plain data.

`ModelShape` fields follow the notation used everywhere else: d model width,
NL layers, H heads, Dh head dim, F FFN width, V vocab, K draft heads (= the
maximum candidate-tree depth), mlp_layers per draft head, T tree nodes with the
root, page size of the paged KV cache.
"""
from __future__ import annotations

from dataclasses import dataclass, replace


@dataclass(frozen=True)
class ModelShape:
    name: str
    d: int
    NL: int
    H: int
    Dh: int
    F: int
    V: int
    dtype: str            # "f32" or "bf16"
    K: int
    mlp_layers: int
    T: int
    batch: tuple
    prompt: tuple
    gen: int
    seed: int
    rms_eps: float = 1e-6
    rope_theta: float = 10000.0
    page: int = 16
    include_root_embedding: int = 1
    medusa: int = 0       # 1: sequentially independent heads on h_last only, first MLP layer residual (the baseline draft head)
    prefix: int = 0       # 1: Hydra++ prefix-attention layer (one extra decoder layer feeding the draft heads)

    def with_(self, **kw) -> "ModelShape":
        return replace(self, **kw)


_BASE_SEED = 0x5EED0000

CONFIGS = {
    1: ModelShape("tiny", 256, 2, 4, 64, 688, 1024, "f32", 3, 1, 16, (1,), (128,), 64, _BASE_SEED + 1),
    2: ModelShape("7b", 4096, 32, 32, 128, 11008, 32000, "bf16", 4, 1, 64, (1,), (512,), 256, _BASE_SEED + 2),
    3: ModelShape("7b++", 4096, 32, 32, 128, 11008, 32000, "bf16", 4, 4, 64, (1, 4, 8, 16), (1024,), 256, _BASE_SEED + 3, prefix=1),
    4: ModelShape("13b", 5120, 40, 40, 128, 13824, 32000, "bf16", 4, 4, 64, (1,), (512, 2048, 4096), 256, _BASE_SEED + 4, prefix=1),
    5: ModelShape("33b", 6656, 60, 52, 128, 17920, 32000, "bf16", 4, 4, 64, (1, 4), (2048,), 256, _BASE_SEED + 5, prefix=1),
}


def get_config(idx: int) -> ModelShape:
    return CONFIGS[idx]
