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


class VerifyAudit:
    """Checks of tree_verify_forward's logits, argmax and margin in the 16-bit family, over all rows of one test.

    Every row, no exemption: argmax is the lowest-index maximum of the library's own logits and margin is their
    top-1 minus top-2, bit for bit (this pins the fused reduction whatever the rounding of the logits).
    Against the oracle: logits within `tol` (max relative error per row); margin within 2 * tol * max|logit|; ids
    exact except on near-tie rows, where a near-tie is an oracle top-2 margin below FOUR TIMES the largest logits
    error measured in this very test (an error e can move the maximum only where the margin is under 2e); such rows
    are counted, the library's pick must still be within that distance of the oracle's maximum, and their share of
    all rows is bounded by `max_skip_frac`."""

    def __init__(self, tol):
        self.tol = tol
        self.rows = []

    def add(self, lib_logits, lib_argmax, lib_margin, ref_logits, ref_argmax):
        lib_logits = np.asarray(lib_logits, dtype=np.float32)
        lib_margin = np.asarray(lib_margin, dtype=np.float32)
        for n in range(lib_logits.shape[0]):
            row = lib_logits[n]
            a = int(np.argmax(row))                                   # numpy returns the first maximum = lowest index
            assert int(lib_argmax[n]) == a, f"row {n}: argmax {int(lib_argmax[n])} is not the lowest-index maximum {a} of the library's logits"
            top2 = np.partition(row, -2)[-2:]                         # [second, first]
            assert np.float32(top2[1] - top2[0]) == lib_margin[n], f"row {n}: margin {lib_margin[n]} != top-1 - top-2 of the library's logits"
            self.rows.append((row.astype(np.float64), int(lib_argmax[n]), float(lib_margin[n]),
                              np.asarray(ref_logits[n], np.float64), int(ref_argmax[n])))

    def finish(self, label, max_skip_frac=0.25):
        err = max(float(np.max(np.abs(g - r)) / np.max(np.abs(r))) for g, _, _, r, _ in self.rows)
        assert err <= self.tol, f"{label}: logits error {err}"
        thr = 4.0 * err
        skipped = 0
        for g, ga, gm, r, ra in self.rows:
            s = np.sort(r)[::-1]
            scale = np.max(np.abs(r))
            assert abs(gm - (s[0] - s[1])) <= 2 * self.tol * scale, f"{label}: margin {gm} vs oracle {s[0] - s[1]}"
            if s[0] - s[1] < thr * scale:
                skipped += 1
                assert r[ga] >= s[0] - thr * scale
            else:
                assert ga == ra, f"{label}: argmax {ga} != oracle {ra} at margin {(s[0] - s[1]) / scale:.2e} (threshold {thr:.2e})"
        n = len(self.rows)
        print(f"{label}: logits err {err:.2e}; near-tie threshold {thr:.2e} of max|logit|; ids exact on {n - skipped} rows, "
              f"{skipped} near-tie rows of {n}", flush=True)
        assert skipped <= max(2, int(max_skip_frac * n)), f"{label}: {skipped} of {n} rows exempt"
        return err, skipped


def generate_checked(make_session, prompt, truth, n_new, model, tol, max_near_ties=2, **gen_kw):
    """Free-running generation on the GPU against the oracle's greedy tokens `truth`, with no way to drop out.

    Where the library's token differs from the oracle's, the oracle's top-2 margin at that position must be a
    near-tie (asserted, counted, at most `max_near_ties`); generation then starts again from the prompt plus the
    oracle's tokens up to and including that position, so that every one of the n_new positions is compared.
    Returns (segments, near_ties); a segment is (first position, tokens that agreed, acceptance lengths, session)."""
    done, near_ties, segments = 0, 0, []
    while done < n_new:
        sess = make_session()
        full = torch.cat([prompt.reshape(-1), torch.tensor(truth[:done], dtype=prompt.dtype)])
        sess.prefill(full.reshape(1, -1))
        toks, accs = sess.generate(n_new - done, **gen_kw)
        assert sess.main.read_flags() == 0
        got = toks[0][:n_new - done]
        want = truth[done:n_new]
        i = next((j for j in range(len(want)) if got[j] != want[j]), None)
        segments.append((done, got if i is None else got[:i], accs, sess))
        if i is None:
            break
        cache = O.FlatCache(model, len(full) + i + 1)
        _, _, _, lg = O.ar_prefill(model, cache, full.tolist() + want[:i])
        assert near_tie(lg, tol), f"token {done + i} differs from the oracle's greedy token and is not a near-tie"
        near_ties += 1
        assert near_ties <= max_near_ties, "too many near-tie divergences"
        done += i + 1
    print(f"generation: {n_new} positions compared, {near_ties} near-tie restarts", flush=True)
    return segments, near_ties
