#!/usr/bin/env python3
"""Decode-step benchmark of lessdec on one MI355X.

A step is one lessdec_step call: one generation step of one attention layer for every
(batch, head) unit of the workload (feature maps, attention over the evicted cache plus
the low-rank terms, H2O score update, eviction, state update, in-place insert).  The
default workload is the Llama-2-7B shape at batch 64 (32 heads, head_dim 128, prompt
1024, 51 heavy + 51 recent slots, rank 8, fp16 cache).  `--layers` independent layer
states are cycled round-robin so the working set (about 1.1 GB) does not fit the 256 MB
Infinity Cache, as in a real 32-layer decode.  Inputs are synthetic and resident in HBM
before the timed region; the state of every layer comes from lessdec_prefill on a
synthetic prompt.

Prints one JSON line: value = unit-steps per second (units x steps / time), ms_per_step,
roofline = algorithmic HBM bytes of the attention launch (the dominant kernel) divided by its
measured time against the 8 TB/s peak, with the same figure for the whole step beside it
(traffic = HBM bytes per launch measured with rocprofv3 counters), cpu_baseline = the fp64
oracle timed on the host cores on a sample of the same workload.  One GPU only.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X published HBM3E bandwidth

# HBM bytes per launch of the attention kernel, from the rocprofv3 FETCH_SIZE / WRITE_SIZE
# counter runs of this same command (profiles/lessdec_step_cfg3_hbm_traffic.txt: counters
# cannot be read from inside the process).  Only for the workload they were taken on.
MEASURED_TRAFFIC_BYTES = {3: 138.6e6}        # the attention launch; the feature-map launch adds 12.1e6


def algorithmic_bytes_per_unit_step(w) -> float:
    """Bytes the method itself must move per unit and step: every retained key and value once,
    the step's rows in and out, the H2O scores and positions, the low-rank state read and
    written, and the per-head feature-map weights shared by the batch rows."""
    e = 2 if w.dtype == "f16" else 4
    C, D, R, Rp, B, G = w.capacity, w.head_dim, w.rank, w.hidden, w.batch, w.q_per_kv
    kv = 2 * C * D * e                       # every retained key and value once
    io = (G + 2) * D * e + G * D * e + 2 * D * e   # q (G heads), k, v in; out (G heads); the inserted pair
    scores = 2 * 8 * C + 4 * C + 4           # acc (fp64) read+write, pos read, one pos write
    state = 2 * (R * D * 4 + R * 8)          # H (fp32) and z (fp64) read + write
    psi = 2 * R * 4                          # psi of the discarded pair read, of the new pair written
    return kv + io + scores + state + psi + _weight_bytes_per_unit_step(w)


def _weight_bytes_per_unit_step(w) -> float:
    """Per-head feature-map weights (phi per query head, psi per key/value head), shared by the batch rows."""
    e = 2 if w.dtype == "f16" else 4
    D, R, Rp, B, G = w.head_dim, w.rank, w.hidden, w.batch, w.q_per_kv
    return ((G + 1) * (D * Rp + Rp * R) + R * R) * e / B


def attend_bytes_per_unit_step(w) -> float:
    """The same figure for the attention launch alone: everything except the weights, which
    only the feature-map launch reads."""
    return algorithmic_bytes_per_unit_step(w) - _weight_bytes_per_unit_step(w)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(w, n_units, n_steps, flags=0):
    """The oracle as it stands, timed on the host cores on a bounded sample of the workload."""
    from oracle import less_oracle as lo
    from paper_2402_09398_amd import workloads as wl
    units = list(range(n_units))
    inp = wl.all_inputs(w.scaled(steps=n_steps), units, workers=16)
    W = wl.head_weights(w)
    st = lo.OracleState(n_units, w.heads, w.head_dim, w.n_heavy, w.n_recent, w.rank, w.hidden, W,
                        flags=flags, head_of_unit=[u % w.heads for u in units], q_per_kv=w.q_per_kv)
    t0 = time.perf_counter()
    st.prefill(inp["Q"], inp["K"], inp["V"], want_out=False)
    t_prefill = time.perf_counter() - t0
    t0 = time.perf_counter()
    for t in range(n_steps):
        st.step(inp["q"][t], inp["k"][t], inp["v"][t])
    t_dec = time.perf_counter() - t0
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": n_units * n_steps / t_dec, "unit": "unit-steps/s", "cores": cores, "kind": "oracle",
            "sample": f"{n_units} units (batch rows 0..{n_units // w.heads - 1}) x {n_steps} decode steps "
                      f"after the oracle's own prompt phase ({t_prefill:.1f} s, not counted)",
            "decode_seconds": t_dec}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4096)
    ap.add_argument("--warmup", type=int, default=128)
    ap.add_argument("--cfg", type=int, default=3, help="workload (1..5), default the batch-64 Llama-2-7B shape")
    ap.add_argument("--layers", type=int, default=8, help="independent layer states cycled round-robin")
    ap.add_argument("--q-per-kv", type=int, default=1,
                    help="G > 1: the workload's heads become heads/G key/value heads with G query heads each "
                         "(multi-query / grouped-query attention); a different workload than the headline one")
    ap.add_argument("--policy", choices=("h2o", "lambda"), default="h2o",
                    help="lambda: Lambda-masking with the paper's split (4 first tokens, the other slots recent); "
                         "a different workload than the headline one")
    ap.add_argument("--prompt-stepwise", action="store_true",
                    help="the sparse policy active from the first prompt token (LESSDEC_FLAG_PROMPT_STEPWISE)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-units", type=int, default=1024)
    ap.add_argument("--cpu-steps", type=int, default=512)
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (every unit is independent; "
                 "sharding would put whole units on each GPU, with no collective). Use --gpus 1.")

    import numpy as np
    import torch
    from paper_2402_09398_amd import LessDec, pack_weights, workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    dev = torch.device("cuda:0")
    w = wl.WORKLOADS[args.cfg]
    if args.q_per_kv > 1:
        if w.heads % args.q_per_kv:
            sys.exit(f"bench.py: --q-per-kv must divide the workload's {w.heads} heads")
        w = w.scaled(name=f"{w.name}-gqa{args.q_per_kv}", heads=w.heads // args.q_per_kv, q_per_kv=args.q_per_kv)
    flags = 0
    if args.policy == "lambda":
        w = w.scaled(name=f"{w.name}-lambda", n_heavy=4, n_recent=w.capacity - 4)
        flags |= 2
    if args.prompt_stepwise:
        w = w.scaled(name=f"{w.name}-prompt-stepwise")
        flags |= 4
    L = args.layers
    U, D, T = w.units, w.head_dim, w.steps

    t0 = time.perf_counter()
    inp = wl.all_inputs(w, workers=16)
    log(f"[bench] inputs for {U} units generated in {time.perf_counter() - t0:.1f} s")
    W = pack_weights(wl.head_weights(w), dev)
    layers = [LessDec(w.batch, w.heads, D, w.n_heavy, w.n_recent, w.rank, w.hidden, w.dtype, W,
                      max_prompt=w.prompt if i == 0 else 0, device=dev, q_per_kv=w.q_per_kv, flags=flags)
              for i in range(L)]
    Q, K, V = (torch.from_numpy(inp[k]).to(dev) for k in ("Q", "K", "V"))
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    pout = torch.empty_like(Q)                               # the prompt's attention outputs are wanted
    layers[0].prefill(Q, K, V, out=pout)                     # warm-up (first launches of its kernels)
    torch.cuda.synchronize()
    e0.record()
    layers[0].prefill(Q, K, V, out=pout)
    e1.record(); torch.cuda.synchronize()
    prefill_ms = e0.elapsed_time(e1)
    # algorithmic flops of the prompt phase per unit: causal Q K^T twice and A V (3 P^2 D), psi of the
    # discarded keys, the state build; the score contractions decide the heavy set and run in fp64
    n_ev = max(w.prompt - w.capacity, 0)
    state_flops = 2.0 * n_ev * (D * w.hidden + w.hidden * w.rank + w.rank ** 2) + 2.0 * w.rank * n_ev * D
    Pn, Cn, G = float(w.prompt), float(w.capacity), float(w.q_per_kv)
    if flags & 2 and flags & 4 and w.prompt > w.capacity:
        # Lambda-masking through the prompt: scores of the cached pairs only, low-rank weights of the
        # discarded ones (phi of every query as well), A V over everything, column sums of the kept tokens
        score_flops = G * (2.0 * Pn * (Cn + 1) * D + Pn ** 2 * w.rank + Pn ** 2 * D + 2.0 * Cn * Pn * D
                           + 2.0 * Pn * (D * w.hidden + w.hidden * w.rank))
        state_flops = 2.0 * Pn * (D * w.hidden + w.hidden * w.rank + w.rank ** 2) + 2.0 * w.rank * n_ev * D
    elif flags & 2:
        score_flops = G * (2.0 * Pn ** 2 * D + 2.0 * Cn * Pn * D)     # the kept set is known: its column sums only
    else:
        score_flops = G * 3.0 * Pn ** 2 * D
    prefill_flops = U * (score_flops + state_flops)
    log(f"[bench] lessdec_prefill P={w.prompt}: {prefill_ms:.1f} ms")
    del Q, K, V, pout
    for lay in layers[1:]:
        for n in lay.STATE:
            getattr(lay, n).copy_(getattr(layers[0], n))
    q, k, v = (torch.from_numpy(inp[n]).to(dev) for n in ("q", "k", "v"))      # [T,U,D]
    del inp
    outs = [torch.empty(q.shape[1:], dtype=layers[0].tdtype, device=dev) for _ in range(L)]
    torch.cuda.synchronize()

    def run(first, count):
        for i in range(first, first + count):
            lay = i % L
            t = ((i // L) + 37 * lay) % T           # every layer walks the token axis at its own offset
            layers[lay].step(q[t], k[t], v[t], outs[lay])

    run(0, args.warmup)
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream()
    e0.record(stream)
    run(args.warmup, args.steps)
    e1.record(stream)
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1)
    ms_per_step = ms / args.steps

    # The two launches of a step, timed one kind at a time on the same stream, same inputs and
    # same layer rotation (the attention launch then reads feature maps of an earlier query,
    # which changes values but not work).
    def run_half(first, count, attend):
        for i in range(first, first + count):
            lay = i % L
            t = ((i // L) + 37 * lay) % T
            if attend:
                layers[lay].step_attend(q[t], k[t], v[t], outs[lay])
            else:
                layers[lay].step_features(q[t], k[t])

    half_ms = {}
    for attend in (False, True):
        run_half(0, args.warmup, attend)
        torch.cuda.synchronize()
        e0.record(stream)
        run_half(args.warmup, args.steps, attend)
        e1.record(stream)
        torch.cuda.synchronize()
        half_ms[attend] = e0.elapsed_time(e1) / args.steps
    attend_bytes = attend_bytes_per_unit_step(w) * U
    attend_achieved = attend_bytes / (half_ms[True] * 1e-3) / 1e9
    unit_steps_per_s = U * args.steps / (ms * 1e-3)
    bytes_per_step = algorithmic_bytes_per_unit_step(w) * U
    achieved = bytes_per_step / (ms_per_step * 1e-3) / 1e9

    result = {
        "metric": "decode steps/sec (batch\u00d7heads) + achieved HBM GB/s vs peak, Llama-2-7B shape",
        "value": unit_steps_per_s,
        "unit": "unit-steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "steps_per_s": 1e3 / ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 storage, f64 scores / f32 values",
        "data": "synthetic",
        "config": {"workload": f"cfg{w.cfg} {w.name}: batch {w.batch} x heads {w.heads} x head_dim {D}, "
                               f"prompt {w.prompt}, {w.n_heavy}+{w.n_recent} slots, rank {w.rank}, hidden {w.hidden}"
                               + (f", {w.q_per_kv} query heads per head" if w.q_per_kv > 1 else "")
                               + (", Lambda-masking" if flags & 2 else "")
                               + (", policy active through the prompt" if flags & 4 else ""),
                   "layers_cycled": L, "prefill_ms": prefill_ms},
        # the prompt phase (secondary path), one warm call: algorithmic flops against the fp64 matrix peak
        "prefill": {"ms": prefill_ms, "prompt_tokens_per_s": U * w.prompt / (prefill_ms * 1e-3),
                    "bound": "mfma", "achieved": prefill_flops / (prefill_ms * 1e-3) / 1e12, "peak": 78.6,
                    "unit": "TFLOP/s", "frac": prefill_flops / (prefill_ms * 1e-3) / 1e12 / 78.6,
                    "flops": prefill_flops,
                    "note": ("algorithmic flops count Q K^T twice (row statistics, column sums) and A V; the "
                             "column sums are computed exactly (fp64) only for tokens that can be kept, found by a "
                             "cheap fp16 pass, and A V runs in fp16, so the figure can exceed the fp64 peak")
                            if not flags & 2 else
                            ("algorithmic flops of this policy: scores in fp64 (all causal pairs, or with the policy "
                             "active through the prompt only the cached ones plus rank-R weights of the discarded "
                             "ones), A V in fp16, column sums of the kept tokens only")},
        # the dominant kernel: the attention launch (lessdec_step_attend), timed by itself
        "roofline": {"bound": "hbm", "achieved": attend_achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": attend_achieved / HBM_PEAK_GBS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(w.cfg) if L >= 8 and w.q_per_kv == 1 and flags == 0 else None,
                     "kernel": ("wpu_step_kernel" if w.q_per_kv == 1 else "gqa_chunk_kernel") + " (lessdec_step_attend)",
                     "bytes_per_launch": attend_bytes, "ms_per_launch": half_ms[True],
                     "features_ms_per_launch": half_ms[False],
                     "whole_step": {"achieved": achieved, "frac": achieved / HBM_PEAK_GBS,
                                    "bytes_per_step": bytes_per_step},
                     "kv_only_frac": 2 * w.capacity * D * (2 if w.dtype == "f16" else 4) * U
                                     / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS},
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, min(args.cpu_units, U), min(args.cpu_steps, T), flags)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
