"""Plumbing shared by the GPU parity tests: the same seeded weights go to the
oracle (CPU, float64) and to the library (device, model dtype)."""
from __future__ import annotations

import numpy as np
import torch

from oracle import hydra_oracle as O
from helpers import make_weights, oracle_model


def gpu_session(cfg, parent, B, max_len, weights, **kw):
    from paper_2402_05109_amd.session import Session
    return Session(cfg, parent, B, max_len, lambda name: weights[name].to("cuda:0"), **kw)


def to_np(t):
    return t.detach().cpu().double().numpy()


def max_rel(got, ref):
    """max_i |got - ref| / max_i |ref| over the last axis, worst row."""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    num = np.max(np.abs(got - ref), axis=-1)
    den = np.maximum(np.max(np.abs(ref), axis=-1), 1e-30)
    return float(np.max(num / den))


def load_oracle_cache(sess, cache_rows, L):
    """Write slots [0, L) of the oracle caches (one per row) into the device pages."""
    if L == 0:
        return
    B = len(cache_rows)
    for l in range(sess.shape.NL):
        plain = np.stack([np.stack([c.K[l, :L], c.V[l, :L]], axis=1) for c in cache_rows])   # [B, L, 2, H, Dh]
        t = torch.tensor(plain, dtype=torch.float32, device="cuda:0").contiguous()
        sess.main.kv_write(B, l, sess.kv, 0, L, t)
    sess.seq_len.fill_(L)
    sess.host_len = L


def read_cache(sess, ctx, first, n):
    """[NL, B, n, 2, H, Dh] float64 of slots first .. first+n-1."""
    s = sess.shape
    out = []
    for l in range(s.NL):
        t = torch.zeros(sess.B, n, 2, s.H, s.Dh, dtype=torch.float32, device="cuda:0")
        ctx.kv_read(sess.B, l, sess.kv, first, n, t)
        out.append(to_np(t))
    return np.stack(out)


def near_tie(logits_row, tol):
    """top-1 minus top-2 of the oracle's logits below tol * max|logits|."""
    s = np.sort(np.asarray(logits_row))[::-1]
    return (s[0] - s[1]) < tol * np.max(np.abs(logits_row))
