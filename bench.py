#!/usr/bin/env python3
"""Benchmark of the Hydra-decoding hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2]

A "step" is one pass of the whole hot path over the batch:
hydra_draft_tree -> tree_verify_forward -> accept_greedy -> kv_compact.
The workload is seeded and synthetic (random-init weights of the named shape,
uniform random prompt); with random heads the natural acceptance length is
about one token per step, so tokens/s is close to steps/s.

Prints ONE JSON line.  `value` is generated tokens per second of the decode loop
with everything resident in HBM.  `roofline` describes the dominant kernel (the
weight-streaming GEMM): algorithmic weight bytes per launch over the HIP-event
duration of the launch.  `cpu_baseline` is the CPU oracle timed on this host on
a bounded sample (see `sample`).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np
import torch


def verify_bytes(cfg, B, L, T):
    """Algorithmic HBM bytes of one tree_verify_forward: every base weight once, the
    cached K/V of the context once, the new K/V written, the token activations."""
    e = 2 if cfg.dtype == "bf16" else 4
    w = e * (cfg.NL * (4 * cfg.d * cfg.d + 3 * cfg.d * cfg.F) + cfg.d * cfg.V)
    kvtok = 2 * cfg.d * cfg.NL * e
    return w + B * ((L + T) * kvtok + T * kvtok) + e * B * T * cfg.d


def draft_bytes(cfg):
    e = 2 if cfg.dtype == "bf16" else 4
    tot = 0
    for i in range(1, cfg.K + 1):
        w1_in = 1 if cfg.medusa else (i + 1 if cfg.include_root_embedding else i)
        tot += e * (w1_in * cfg.d * cfg.d + (cfg.mlp_layers - 1) * cfg.d * cfg.d + cfg.d * cfg.V)
    return tot


def read_traffic(config):
    """HBM bytes per GEMM launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (see profiles/), and where the
    figure comes from: counters cannot be read inside this run, so the committed summary is quoted together with the
    commit that last touched it (a summary older than the kernels it describes is visible that way)."""
    name = f"gemm_bf16_kernel_config{config}_traffic.txt"
    path = os.path.join(ROOT, "profiles", name)
    try:
        val, when = None, None
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                val = float(line.split(":")[1])
            if line.startswith("collected:"):
                when = line.split(":", 1)[1].strip()
        if val is None:
            return None, None
        src = f"profiles/{name}" + (f", collected {when}" if when else "")
        try:
            import subprocess
            r = subprocess.run(["git", "-C", ROOT, "log", "-1", "--format=%h %cs", "--", f"profiles/{name}"], capture_output=True, text=True, timeout=10)
            if r.returncode == 0 and r.stdout.strip():
                src += f" (last changed in commit {r.stdout.strip()})"
        except Exception:
            pass
        return val, src
    except OSError:
        return None, None


def cpu_baseline(cfg, parent, L, n_layers_sample, get_cpu, threads=None):
    """Oracle on the host cores: one Hydra step (draft + verify) of the same shape with
    `n_layers_sample` of the NL decoder layers, layer time scaled to NL.  threads: limit of the BLAS thread pool
    (None = all it takes by itself)."""
    if threads is not None:
        import threadpoolctl
        with threadpoolctl.threadpool_limits(limits=threads):
            return cpu_baseline(cfg, parent, L, n_layers_sample, get_cpu)
    from oracle import hydra_oracle as O
    tree = O.Tree(parent)
    names = ["embed", "lm_head", "final_norm"]
    for l in range(n_layers_sample):
        names += [f"layers.{l}.{t}" for t in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")]
    for i in range(1, cfg.K + 1):
        names += [f"heads.{i}.w1", f"heads.{i}.b1", f"heads.{i}.wout"]
        for j in range(2, cfg.mlp_layers + 1):
            names += [f"heads.{i}.w{j}", f"heads.{i}.b{j}"]
    W = {n: get_cpu(n) for n in names}
    m = O.Model(cfg.d, n_layers_sample, cfg.H, cfg.Dh, cfg.F, cfg.V, cfg.K, cfg.mlp_layers, W,
                rms_eps=cfg.rms_eps, rope_theta=cfg.rope_theta, include_root_embedding=cfg.include_root_embedding)
    rng = np.random.default_rng(0)
    cache = O.FlatCache(m, L + tree.T)
    cache.K[:, :L] = rng.standard_normal(cache.K[:, :L].shape) * 0.5
    cache.V[:, :L] = rng.standard_normal(cache.V[:, :L].shape) * 0.5
    h = rng.standard_normal(cfg.d)
    t0 = time.perf_counter()
    tok, _ = O.draft_tree(m, tree, h, 1)
    t_draft = time.perf_counter() - t0
    # time the LM head + embedding part separately by a zero-layer model
    m0 = O.Model(cfg.d, 0, cfg.H, cfg.Dh, cfg.F, cfg.V, cfg.K, cfg.mlp_layers, W, rms_eps=cfg.rms_eps, rope_theta=cfg.rope_theta)
    t0 = time.perf_counter()
    O.tree_verify(m0, O.FlatCache(m0, L + tree.T), L, tree, tok)
    t_head = time.perf_counter() - t0
    t0 = time.perf_counter()
    O.tree_verify(m, cache, L, tree, tok)
    t_verify_s = time.perf_counter() - t0
    per_layer = max(t_verify_s - t_head, 0.0) / n_layers_sample
    t_step = t_draft + t_head + per_layer * cfg.NL
    return t_step, t_draft + t_head + t_verify_s


MFMA_PEAK_TFLOPS = 2500.0          # dense 16-bit matrix-core peak of MI355X (the contractions run mfma_f32_32x32x16_f16)


def verify_flops(cfg, B, T):
    """Multiply-adds x 2 of the weight contractions of one tree_verify_forward over B * T rows."""
    return 2.0 * B * T * (cfg.NL * (4 * cfg.d * cfg.d + 3 * cfg.d * cfg.F) + cfg.d * cfg.V)


def rooflines(cfg, B, L, T, ms):
    """Both rooflines of a verify step: HBM (algorithmic bytes over 8 TB/s) and matrix cores (flops over 2.5 PFLOP/s);
    the one whose floor is higher bounds the step (paper, section 6.2: large batch x tree makes verification compute-bound)."""
    vb, fl = verify_bytes(cfg, B, L, T), verify_flops(cfg, B, T)
    hbm_floor, mfma_floor = vb / 8e12 * 1e3, fl / (MFMA_PEAK_TFLOPS * 1e12) * 1e3
    return {"rows": B * T, "ms": ms, "algorithmic_GB": vb / 1e9, "GBps": vb / (ms * 1e-3) / 1e9, "frac_of_8TBps": vb / (ms * 1e-3) / 8e12,
            "TFLOPs": fl / (ms * 1e-3) / 1e12, "frac_of_mfma_peak": fl / (ms * 1e-3) / (MFMA_PEAK_TFLOPS * 1e12),
            "bound": "mfma" if mfma_floor > hbm_floor else "hbm", "floor_ms": max(hbm_floor, mfma_floor)}


def other_configs(budget_s, dev, reps=20):
    """Verify-step latency and roofline fractions of the other workload configurations (3: 7B shape with Hydra++
    heads at batch 1..16 and prompt 1024; 4: 13B shape at contexts 512 / 2048 / 4096; 5: 33B shape at batch 1 and 4,
    context 2048), each on a session of its own with seeded weights.  The cache content does not influence the time
    of a step, so the context is set, not prefilled.  Stops opening new sessions once the time budget is used up."""
    from synth import CONFIGS, WeightSpec, frozen_tree, make_tensor
    from paper_2402_05109_amd.session import Session
    plan = [(3, B, (1024,)) for B in (1, 4, 8, 16)] + [(4, 1, (512, 2048, 4096))] + [(5, 1, (2048,)), (5, 4, (2048,))]
    t_start, rows, skipped = time.perf_counter(), [], []
    for idx, B, contexts in plan:
        if time.perf_counter() - t_start > budget_s:
            skipped.append(f"config {idx} B={B}")
            continue
        cfg = CONFIGS[idx]
        spec = WeightSpec(cfg)
        parent = frozen_tree("prior64")
        sess = Session(cfg, parent, B, max(contexts) + 2 * cfg.T, lambda n: make_tensor(spec, n, device=dev), device=dev, prefill_chunk=64)
        for L in contexts:
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            ts = []
            for i in range(3 + reps):
                sess.seq_len.fill_(L); sess.host_len = L
                ev0.record(); sess.verify(); ev1.record(); ev1.synchronize()
                if i >= 3:
                    ts.append(ev0.elapsed_time(ev1))
            r = rooflines(cfg, B, L, cfg.T, float(np.median(ts)))
            r.update({"config": idx, "shape": cfg.name, "B": B, "T": cfg.T, "context": L, "device_flags": sess.main.read_flags()})
            rows.append(r)
        stage(f"config {idx} B={B} measured")
        del sess
        torch.cuda.empty_cache()
    return {"what": "tree_verify_forward, median of %d calls (HIP events), seeded weights, context set not prefilled" % reps,
            "rows": rows, "skipped_for_time": skipped}


SWEEP_T = (1, 2, 4, 6, 8, 12, 16, 24, 32, 48, 64, 96, 128)
SWEEP_B = (1, 2, 4, 8, 16)


def tree_sweep(cfg, L0, steps, dev):
    """Tree-size sweep (paper, section 4 "Discovering performant decoding trees" and the appendix on optimal trees):
    proposal trees T_1 .. T_128 grown greedily under a synthetic acceptance model, one whole step (draft, verify,
    accept, compact) timed for a ladder of sizes and batch sizes, and per batch size the size with the highest
    expected tokens/s = B * E[acceptance length](T) / step time.  The expectation is a property of the synthetic
    prior (synth/trees.py), not of a corpus; the step times are measured."""
    from synth import WeightSpec, expected_acceptance, make_tensor, proposal_trees
    from paper_2402_05109_amd.session import Session
    trees = proposal_trees(max(SWEEP_T))
    exp = {T: float(expected_acceptance(trees[T - 1])) for T in SWEEP_T}
    spec = WeightSpec(cfg)
    rows = []
    for B in SWEEP_B:
        sess = Session(cfg, trees[SWEEP_T[0] - 1], B, L0 + max(SWEEP_T) + 64, lambda n: make_tensor(spec, n, device=dev), device=dev, prefill_chunk=64)
        names = {SWEEP_T[0]: "main"}
        for T in SWEEP_T[1:]:
            names[T] = f"tree{T}"
            sess.add_tree(names[T], trees[T - 1])
        per_T = []
        for T in SWEEP_T:
            nm = names[T]
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            ts = []
            for i in range(3 + steps):
                sess.seq_len.fill_(L0); sess.host_len = L0              # cache content is irrelevant to the time of a step
                ev0.record(); sess.step(nm); ev1.record(); ev1.synchronize()
                if i >= 3:
                    ts.append(ev0.elapsed_time(ev1))
            ms = float(np.median(ts))
            per_T.append({"T": T, "ms_per_step": ms, "expected_acceptance": exp[T], "tokens_per_s_expected": B * exp[T] / (ms * 1e-3)})
        assert sess.main.read_flags() == 0
        best = max(per_T, key=lambda r: r["tokens_per_s_expected"])
        rows.append({"B": B, "best_T": best["T"], "tokens_per_s_expected": best["tokens_per_s_expected"],
                     "ms_per_step_at_best": best["ms_per_step"], "autoregressive_tokens_per_s": per_T[0]["tokens_per_s_expected"], "per_T": per_T})
        stage(f"tree sweep, batch {B}: best T = {best['T']}")
        del sess
        torch.cuda.empty_cache()
    return {"prior": "synthetic acceptance model q(depth j, rank r) = 0.3 * 0.8^(j-1) * 0.5^r, not corpus statistics",
            "context": L0, "sizes": list(SWEEP_T), "rows": rows}


def layer_kernel_timeline(cfg, L, dev, layers=8):
    """Where the time goes inside the persistent layer kernel (HYDRA_LAYER_KERNEL=1): wall-clock stamps that every
    workgroup leaves per step and layer, reduced to per-step figures (mean over the inner layers).  Also times the same
    verify call with separate launches.  The model is cut to `layers` decoder layers (the stamps of all workgroups of
    32 layers are not needed for a per-layer figure)."""
    import numpy as np
    from synth import WeightSpec, frozen_tree, make_tensor, uniform_tokens
    from paper_2402_05109_amd.session import Session
    cfg = cfg.with_(NL=layers, K=1)
    spec = WeightSpec(cfg)
    parent = frozen_tree({16: "tiny16", 32: "prior32", 64: "prior64", 128: "prior128"}[cfg.T])
    T = len(parent)

    def timed(env):
        for k in ("HYDRA_LAYER_KERNEL", "HYDRA_LAYER_KERNEL_STAMPS"):
            os.environ.pop(k, None)
        os.environ.update(env)
        sess = Session(cfg, parent, 1, L + 64, lambda n: make_tensor(spec, n, device=dev), device=dev, prefill_chunk=64)
        sess.out().tree_tokens.copy_(uniform_tokens(99, 0, T, cfg.V).reshape(1, -1).to(torch.int32))
        sess.seq_len.fill_(L)
        sess.host_len = L
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ts = []
        for _ in range(12):
            sess.seq_len.fill_(L)
            e0.record(); sess.verify(); e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        return sess, sorted(ts[2:])[5]

    _, ms_launches = timed({})
    sess, ms_kernel = timed({"HYDRA_LAYER_KERNEL": "1", "HYDRA_LAYER_KERNEL_STAMPS": "1"})
    info = sess.main.layer_kernel_info(1)          # eligible, byte offset of the stamps in the workspace, workgroups, steps
    if not info[0]:
        return {"error": "the layer kernel does not take this shape"}
    G, NS = info[2], info[3]
    st = sess.ws[info[1]:info[1] + layers * NS * G * 8 * 8].view(torch.int64).cpu().numpy().reshape(layers, NS, G, 8).astype(np.float64) * 0.01
    flags = sess.main.read_flags()
    names = ["q|k|v GEMM + RoPE + cache append", "tree attention", "O GEMM", "residual + norm 1", "gate/up GEMM + SwiGLU", "down GEMM", "residual + norm 2"]
    steps, per_layer = [], 0.0
    for s in range(NS):
        rows = []
        for l in range(1, layers - 1):
            b, e, a, r = st[l, s, :, 0], st[l, s, :, 1], st[l, s, :, 2], st[l, s, :, 3]      # begin, work done, counted in, released
            work = e - b
            gemm = s in (0, 2, 4, 5)
            q = st[l, s]
            if gemm:    # GEMM steps also stamp: first X tile in, last MFMA, stores issued (only workgroups with an item write them)
                busy = (q[:, 4] >= b) & (q[:, 5] >= q[:, 4]) & (q[:, 6] >= q[:, 5]) & (q[:, 6] <= e)
            else:
                busy = work > 1.0
            n = int(busy.sum())
            row = [n, work[busy].mean() if n else 0.0, work.max(), a.max() - e.max(), r.max() - a.max(), r.max() - b.min()]
            if gemm:
                row += [(q[busy, 4] - q[busy, 0]).mean(), (q[busy, 5] - q[busy, 4]).mean(), (q[busy, 6] - q[busy, 5]).mean(), (q[busy, 1] - q[busy, 6]).mean()] if n else [0.0] * 4
            rows.append(row)
        m = np.mean(np.array(rows), axis=0)
        d = {"step": names[s], "busy_workgroups": int(round(m[0])), "work_us_mean": round(m[1], 2), "work_us_slowest": round(m[2], 2),
             "last_work_to_last_arrival_us": round(m[3], 2), "last_arrival_to_last_release_us": round(m[4], 2), "span_us": round(m[5], 2)}
        if len(m) > 6:
            d.update({"wait_for_input_us": round(m[6], 2), "stream_us": round(m[7], 2), "reduce_and_epilogue_us": round(m[8], 2),
                      "stores_acknowledged_us": round(m[9], 2)})
        per_layer += m[5]
        steps.append(d)
    return {"what": f"one tree_verify_forward of {layers} layers at context {L}, T = {T}: separate launches against the persistent layer kernel; "
                    "per-step figures are means over the inner layers of in-kernel wall-clock stamps (100 MHz counter)",
            "ms_separate_launches": round(ms_launches, 4), "ms_layer_kernel": round(ms_kernel, 4),
            "us_per_layer_in_layer_kernel": round(per_layer, 2), "device_flags": int(flags), "steps": steps}


def stage(msg):
    """one progress line per finished stage, on stderr (stdout carries only the JSON line)"""
    print(f"bench.py: {msg}", file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--tree", type=int, default=0, choices=[0, 16, 32, 64, 128],
                    help="candidate-tree size (nodes with the root); 0 = the configuration's own (the headline workload)")
    ap.add_argument("--batch", type=int, default=0, help="batch rows (0 = the configuration's first batch size)")
    ap.add_argument("--prompt", type=int, default=0, help="prompt length (0 = the configuration's first prompt length)")
    ap.add_argument("--medusa", action="store_true",
                    help="Medusa-style draft heads (h_last only, one hidden layer with a skip connection) instead of Hydra heads: the baseline draft cost")
    ap.add_argument("--typical", action="store_true",
                    help="also time accept_typical (tau 0.7, eps 0.15, alpha sqrt(eps)); the session then keeps the [B,T,V] logits")
    ap.add_argument("--sweep", action="store_true",
                    help="only the tree-size sweep: step time for proposal trees of 1..128 nodes at batch 1..16 and the size of highest expected tokens/s per batch size")
    ap.add_argument("--layer-kernel-timeline", action="store_true",
                    help="only the in-kernel timeline of the persistent layer kernel (opt-in path, HYDRA_LAYER_KERNEL=1) against separate launches, on 8 layers")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--other-configs-budget", type=float, default=75.0,
                    help="seconds the default run may spend on the verify-step figures of configs 3, 4 and 5 (0 = skip them)")
    ap.add_argument("--no-injected", action="store_true",
                    help="skip the injected-acceptance points (for counter-collection runs, where every launch is slow)")
    ap.add_argument("--layers", type=int, default=0, help="debug: override the number of layers (invalidates the result)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path shards by batch row with no collectives, "
              "so N GPUs are N independent copies of this run); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    if not os.path.exists(os.path.join(ROOT, "paper_2402_05109_amd", "libhydra.so")):      # nothing built yet: build, then load
        from paper_2402_05109_amd.build import build_library
        build_library(verbose=False)
    from synth import CONFIGS, WeightSpec, frozen_tree, make_tensor, uniform_tokens
    from paper_2402_05109_amd.session import Session

    cfg = CONFIGS[args.config]
    if args.layers:
        cfg = cfg.with_(NL=args.layers)
    if args.sweep:
        sw = tree_sweep(cfg, args.prompt or cfg.prompt[0], 8, "cuda:0")
        print(json.dumps({"metric": "tree-size sweep: expected tokens/s per (T, B)", "unit": "tokens/s", "n_gpus": 1, "data": "synthetic",
                          "config": {"workload": f"config {args.config}: {cfg.name} shape, {cfg.K} heads x {cfg.mlp_layers}-layer MLP, proposal trees of "
                                                 f"{SWEEP_T[0]}..{SWEEP_T[-1]} nodes, B in {list(SWEEP_B)}, context {args.prompt or cfg.prompt[0]}"},
                          "tree_sweep": sw}))
        return
    if args.tree:
        cfg = cfg.with_(T=args.tree)
    if args.layer_kernel_timeline:
        tl = layer_kernel_timeline(cfg, (args.prompt or cfg.prompt[0]) + 11, "cuda:0")
        print(json.dumps({"metric": "in-kernel timeline of the persistent layer kernel", "unit": "us", "n_gpus": 1, "data": "synthetic",
                          "config": {"workload": f"config {args.config}: {cfg.name} shape, T={cfg.T}, B=1"}, "layer_kernel_timeline": tl}))
        return
    if args.medusa:
        cfg = cfg.with_(medusa=1)
    tree_name = {16: "tiny16", 32: "prior32", 64: "prior64", 128: "prior128"}[cfg.T]
    parent = frozen_tree(tree_name)
    B, L0 = (args.batch or cfg.batch[0]), (args.prompt or cfg.prompt[0])
    spec = WeightSpec(cfg)
    dev = "cuda:0"
    max_len = L0 + (args.steps + args.warmup + 8 + 3 * 40) * (cfg.K + 1) + 2 * cfg.T
    sess = Session(cfg, parent, B, max_len, lambda n: make_tensor(spec, n, device=dev), device=dev, prefill_chunk=128,
                   want_logits=args.typical)
    stage("weights packed on the device")
    prompts = torch.stack([uniform_tokens(cfg.seed, b, L0, cfg.V) for b in range(B)])
    sess.prefill(prompts)
    torch.cuda.synchronize()
    stage("prompt prefilled")

    o = sess.out()
    acc_log = torch.zeros(args.steps, B, dtype=torch.int32, device=dev)
    for _ in range(args.warmup):
        sess.step()
    sess.sync_len()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        sess.step()
        acc_log[i].copy_(o.n_acc)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    tokens = int(acc_log.sum().item())
    flags = sess.main.read_flags()
    stage(f"{args.steps} timed steps done")
    L_end = sess.sync_len()

    # per-call latencies at the end-of-run context length (seq_len restored after each step)
    def snapshot():
        return (sess.seq_len.clone(), sess.h_last.clone(), sess.root.clone(), sess.host_len,
                sess.pseq_len.clone() if sess.prefix else None)

    def restore(saved):
        sess.seq_len.copy_(saved[0]); sess.h_last.copy_(saved[1]); sess.root.copy_(saved[2]); sess.host_len = saved[3]
        if sess.prefix:
            sess.pseq_len.copy_(saved[4])

    def timed(fn, reps=50):
        saved = snapshot()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ts = []
        for _ in range(reps):
            ev0.record(); fn(); ev1.record(); ev1.synchronize()
            ts.append(ev0.elapsed_time(ev1))
            restore(saved)
        return float(np.median(ts))

    t_draft = timed(sess.draft)
    t_verify = timed(sess.verify)
    t_tail = timed(lambda: (sess.accept(), sess.compact()))
    t_prefix = timed(sess.prefix_attention) if sess.prefix else None
    t_typical = None
    typical_loop = None
    if args.typical:
        u_dev = torch.rand(B, device=dev)
        t_typical = timed(lambda: sess.accept_typical(0.7, 0.15, 0.15 ** 0.5, u_dev))
        # the whole loop under the typical criterion (section 6.3's setting: tau 0.7, eps 0.15, alpha sqrt(eps)): draft ->
        # verify (keeps the [B,T,V] logits) -> accept_typical with a fresh uniform number per row -> compact
        saved = snapshot()
        n_typ = 32
        us = torch.rand(n_typ, B, device=dev)
        acc_t = torch.zeros(n_typ, B, dtype=torch.int32, device=dev)
        sess.step(typical=(0.7, 0.15, 0.15 ** 0.5, us[0]))
        restore(saved)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n_typ):
            sess.step(typical=(0.7, 0.15, 0.15 ** 0.5, us[i]))
            acc_t[i].copy_(o.n_acc)
        torch.cuda.synchronize()
        dt_t = time.perf_counter() - t0
        tok_t = int(acc_t.sum().item())
        typical_loop = {"steps": n_typ, "ms_per_step": dt_t / n_typ * 1e3, "tokens_per_s": tok_t / dt_t, "mean_acceptance": tok_t / (n_typ * B),
                        "tau": 0.7, "eps": 0.15, "alpha": 0.15 ** 0.5,
                        "note": "with random-init weights the logits are nearly flat, so nearly every candidate passes this criterion: the acceptance "
                                "length is an artefact of the synthetic weights; the step time is real"}
        restore(saved)
        sess.sync_len()
    vb = verify_bytes(cfg, B, L_end, cfg.T)

    # dominant kernel: the weight-streaming GEMM.  HIP events (recorded by the library on the launch stream)
    # around every GEMM launch of 8 tree_verify_forward calls at the end-of-run context length.
    saved = snapshot()
    sess.main.profile_begin()
    for _ in range(8):
        sess.verify()
    n_launch, ms_sum, w_bytes = sess.main.profile_end()
    restore(saved)
    stage("per-call timings done")
    peak = 8000.0
    ach = (w_bytes / n_launch) / (ms_sum / n_launch * 1e-3) / 1e9 if n_launch else 0.0
    traffic, traffic_src = read_traffic(args.config)
    # throughput at injected acceptance lengths: between verify and accept, the base model's greedy token at the
    # first j nodes of the left-most root-to-leaf path is overwritten with the drafted child token, so accept_greedy
    # returns a fixed length (the generated text is then meaningless; only the cost of the step is real)
    injected = []
    kids = {}
    for n, pa in enumerate(parent):
        if pa >= 0 and pa not in kids:
            kids[pa] = n
    chain = [0]
    while chain[-1] in kids:
        chain.append(kids[chain[-1]])
    sess.sync_len()
    for a in sorted({2, 3, len(chain)}):
        if args.no_injected or a > len(chain) or sess.host_len + 40 * a + cfg.T + 8 > max_len:
            continue
        src = torch.tensor(chain[1:a], dtype=torch.long, device=dev)
        dst = torch.tensor(chain[:a - 1], dtype=torch.long, device=dev)
        n_steps = 32
        o.argmax[:, dst] = o.tree_tokens[:, src]           # untimed: first use of the indexing kernels
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n_steps):
            sess.draft(); sess.verify()
            o.argmax[:, dst] = o.tree_tokens[:, src]
            if a < len(chain):
                o.argmax[:, chain[a - 1]] = 1          # end of the injected path (a drafted child equal to token 1 is a 1-in-V accident)
            sess.accept()
            pre = sess.host_len
            sess.compact()
            if sess.prefix:
                post, sess.host_len = sess.host_len, pre
                sess.prefix_attention()
                sess.host_len = post
        torch.cuda.synchronize()
        t = (time.perf_counter() - t0) / n_steps
        injected.append({"accept_len": a, "ms_per_step": t * 1e3, "tokens_per_s": a * B / t, "n_acc_check": int(o.n_acc[0])})
        sess.sync_len()
        stage(f"injected acceptance length {a} done")

    # autoregressive baseline with the same kernels (one-node tree)
    sess.ctx("ar")
    t_ar = timed(lambda: sess.step("ar"))

    out = {
        "metric": "generated tokens/s at batch 1, 7B shape; verify-step HBM GB/s vs peak" if args.config == 2 else f"generated tokens/s, config {args.config}",
        "value": tokens / dt, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 weights, f16 activations and KV cache, f32 accumulation" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"config {args.config}: {cfg.name} shape d={cfg.d} NL={cfg.NL} H={cfg.H}x{cfg.Dh} F={cfg.F} V={cfg.V}, "
                               f"{cfg.K} {'Medusa-style' if cfg.medusa else 'Hydra'} heads x {cfg.mlp_layers}-layer MLP{' + prefix-attention layer' if cfg.prefix else ''}, tree {tree_name} (T={cfg.T}), B={B}, "
                               f"prompt {L0} uniform tokens, paged KV (16), natural acceptance",
                   "tokens_generated": tokens, "mean_acceptance": tokens / (args.steps * B), "context_at_end": L_end,
                   "device_flags": flags},
        "verify": {"ms": t_verify, "algorithmic_GB": vb / 1e9, "GBps": vb / (t_verify * 1e-3) / 1e9,
                   "frac_of_8TBps": vb / (t_verify * 1e-3) / 8e12, "context": L_end},
        "draft": {"ms": t_draft, "algorithmic_GB": draft_bytes(cfg) / 1e9, "GBps": draft_bytes(cfg) / (t_draft * 1e-3) / 1e9},
        "accept_compact_ms": t_tail,
        "prefix_attention_ms": t_prefix,
        "accept_typical_ms": t_typical,
        "typical_acceptance_loop": typical_loop,
        "autoregressive_same_kernels": {"ms_per_token": t_ar, "tokens_per_s": 1e3 / t_ar * B},
        "injected_acceptance": injected,
        "roofline": {"bound": "hbm", "kernel": "gemm_bf16_kernel" if cfg.dtype == "bf16" else "gemm_f32_kernel",
                     "achieved": ach, "peak": peak, "unit": "GB/s", "frac": ach / peak, "traffic": traffic, "traffic_source": traffic_src,
                     "launches_timed": n_launch, "avg_launch_us": ms_sum / max(n_launch, 1) * 1e3,
                     "algorithmic_bytes_per_launch": w_bytes / max(n_launch, 1),
                     "timing": "HIP events attached to each launch on its stream (they take the kernel's own begin and end times)",
                     "scope": "the 129 GEMM launches of one tree_verify_forward (4 per layer + LM head), averaged over 8 calls"},
    }
    stage("injected-acceptance points done")
    out["verify"].update({k: v for k, v in rooflines(cfg, B, L_end, cfg.T, t_verify).items() if k in ("rows", "TFLOPs", "frac_of_mfma_peak", "bound", "floor_ms")})
    if args.other_configs_budget > 0 and args.config == 2 and not args.layers:
        del sess
        torch.cuda.empty_cache()
        out["other_configs"] = other_configs(args.other_configs_budget, dev)
    if not args.no_cpu_baseline:
        ns = min(8, cfg.NL)
        cores = os.cpu_count() or 1
        try:
            import threadpoolctl
            info = threadpoolctl.threadpool_info()
            cores = max([i.get("num_threads", 1) for i in info] + [1])
        except Exception:
            pass
        cpu = lambda n: make_tensor(spec, n, device=dev).cpu()
        t_step, t_spent = cpu_baseline(cfg, parent, L0, ns, cpu)
        out["cpu_baseline"] = {"value": B / t_step, "unit": "tokens/s", "cores": cores, "kind": "oracle",
                               "sample": f"one Hydra step (all {cfg.K} draft heads, LM head, T={cfg.T} tree, context {L0}) with "
                                         f"{ns} of {cfg.NL} decoder layers timed ({t_spent:.1f} s of CPU work) and the per-layer time "
                                         f"scaled to {cfg.NL} layers; acceptance 1 token/step"}
        stage("oracle timed on all threads")
        try:
            ns1 = min(1, cfg.NL)
            t_step1, t_spent1 = cpu_baseline(cfg, parent, L0, ns1, cpu, threads=1)
            out["cpu_baseline"]["one_thread"] = {"value": B / t_step1, "unit": "tokens/s", "cores": 1,
                                                 "sample": f"the same step with {ns1} of {cfg.NL} decoder layers timed on one thread ({t_spent1:.1f} s of CPU work), scaled the same way"}
            stage("oracle timed on one thread")
        except Exception as e:                     # no thread-pool control on this host: the all-threads figure stands alone
            out["cpu_baseline"]["one_thread"] = {"value": None, "note": f"not measured: {e}"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
