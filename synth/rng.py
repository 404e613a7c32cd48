"""Counter-based, integer-exact random numbers written with torch integer ops.

The same code runs on a CPU tensor and on a GPU tensor and gives the same bits,
because every step is 64-bit integer arithmetic (wrapping multiply, xor, shifts)
followed by ONE correctly rounded fp32 multiply.  No transcendental functions.

Stream definition, for a (seed, tensor_id) pair and element index e:
    key  = mix64(seed * P1 + tensor_id * P2 + P3)
    z_r  = mix64(key + (3 e + r) * GOLDEN),        r = 0, 1, 2
    s    = sum of the four 16-bit fields of z_0, z_1, z_2        (12 fields)
    x    = fp32(s - 393210) * fp32(std / 65536)
The sum of 12 independent uniform 16-bit integers has mean 12 * 32767.5 = 393210
and standard deviation 65536 (to 1e-10 relative), so x is an Irwin-Hall(12)
approximation of N(0, std^2), bounded at +-6 std.
"""
from __future__ import annotations

import torch

_MASK64 = (1 << 64) - 1


def _s64(v: int) -> int:
    """Python int (mod 2^64) -> the signed value torch.int64 holds for it."""
    v &= _MASK64
    return v - (1 << 64) if v >= (1 << 63) else v


_GOLDEN = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB
_P1 = 0xD6E8FEB86659FD93
_P2 = 0xA0761D6478BD642F
_P3 = 0xE7037ED1A0B428DB


def _mix64_int(z: int) -> int:
    z &= _MASK64
    z = ((z ^ (z >> 30)) * _C1) & _MASK64
    z = ((z ^ (z >> 27)) * _C2) & _MASK64
    return z ^ (z >> 31)


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right of an int64 tensor."""
    return (z >> s) & ((1 << (64 - s)) - 1)


def _mix64(z: torch.Tensor) -> torch.Tensor:
    z = (z ^ _lsr(z, 30)) * _s64(_C1)
    z = (z ^ _lsr(z, 27)) * _s64(_C2)
    return z ^ _lsr(z, 31)


def stream_key(seed: int, tensor_id: int) -> int:
    return _mix64_int(seed * _P1 + tensor_id * _P2 + _P3)


def _fields_sum(z: torch.Tensor) -> torch.Tensor:
    return (z & 0xFFFF) + (_lsr(z, 16) & 0xFFFF) + (_lsr(z, 32) & 0xFFFF) + _lsr(z, 48)


def _irwin_hall_sum(key: int, start: int, count: int, device) -> torch.Tensor:
    e = torch.arange(start, start + count, dtype=torch.int64, device=device)
    base = e * _s64(3 * _GOLDEN) + _s64(key)
    s = _fields_sum(_mix64(base))
    s += _fields_sum(_mix64(base + _s64(_GOLDEN)))
    s += _fields_sum(_mix64(base + _s64(2 * _GOLDEN)))
    return s


def normal_tensor(seed: int, tensor_id: int, shape, std: float = 0.02,
                  dtype: torch.dtype = torch.float32, device="cpu",
                  chunk: int = 1 << 24) -> torch.Tensor:
    """Tensor of the given shape, ~N(0, std^2), bit-identical on CPU and GPU.

    dtype float32 gives the fp32 value; bfloat16 gives that value rounded to
    nearest-even (torch's conversion), the form bf16 configurations consume.
    """
    n = 1
    for v in shape:
        n *= int(v)
    key = stream_key(seed, tensor_id)
    out = torch.empty(n, dtype=dtype, device=device)
    scale = torch.tensor(std / 65536.0, dtype=torch.float32, device=device)
    for start in range(0, n, chunk):
        cnt = min(chunk, n - start)
        s = _irwin_hall_sum(key, start, cnt, device)
        x = (s - 393210).to(torch.float32) * scale
        out[start:start + cnt] = x.to(dtype)
    return out.reshape(*shape)


def uniform_tokens(seed: int, stream_id: int, count: int, vocab: int,
                   device="cpu") -> torch.Tensor:
    """`count` token ids, i.i.d. uniform on [0, vocab) (int32)."""
    key = stream_key(seed ^ 0x70726F6D7074, stream_id)
    e = torch.arange(count, dtype=torch.int64, device=device)
    z = _mix64(e * _s64(_GOLDEN) + _s64(key))
    return (_lsr(z, 11) % vocab).to(torch.int32)


def uniform_ints(seed: int, stream_id: int, count: int, modulus: int) -> list:
    """Small helper for seeded structural choices (random trees, depths)."""
    key = stream_key(seed ^ 0x7472656573, stream_id)
    return [(_mix64_int(key + i * _GOLDEN) >> 11) % modulus for i in range(count)]
