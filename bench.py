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
roofline = the method's algorithmic HBM bytes per step divided by the measured time of a step
(one launch on the headline workload: the feature-map jobs run inside the attention launch)
against the 8 TB/s peak, beside it the same against the read rate a probe kernel sustains on
this chip, the step timed again as replays of a HIP graph (median and minimum), the bytes this
implementation moves on top of the algorithmic ones, and traffic = HBM bytes per step measured
with rocprofv3 counters; cpu_baseline = the fp64 oracle timed on the host cores on a sample of
the same workload.  One GPU only.
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

# HBM bytes per step (both directions), from the rocprofv3 FETCH_SIZE / WRITE_SIZE counter runs of
# this same command on this build (profiles/lessdec_step_cfg3_hbm_traffic.txt: counters cannot be
# read from inside the process).  Only for the workload and launch shape they were taken on.
MEASURED_TRAFFIC_BYTES = {3: 147.8e6}        # 132.0 MB read + 15.8 MB written by the one launch of a step


def algorithmic_bytes_per_unit_step(w) -> float:
    """Bytes the method itself must move per unit and step: every retained key and value once,
    the step's rows in and out, the inserted pair, the H2O scores (4-byte) read and written, the
    positions, the low-rank state (4-byte) read and written, psi of the discarded and of the new
    pair, and the per-head feature-map weights shared by the batch rows."""
    e = 2 if w.dtype == "f16" else 4
    C, D, R, Rp, B, G = w.capacity, w.head_dim, w.rank, w.hidden, w.batch, w.q_per_kv
    kv = 2 * C * D * e                       # every retained key and value once
    io = (G + 2) * D * e + G * D * e + 2 * D * e   # q (G heads), k, v in; out (G heads); the inserted pair
    scores = 2 * 4 * C + 4 * C + 4           # acc read+write, pos read, one pos write
    state = 2 * (R * D + R) * 4              # H and z read + write
    psi = 2 * R * 4                          # psi of the discarded pair read, of the new pair written
    weights = ((G + 1) * (D * Rp + Rp * R) + R * R) * e / B
    return kv + io + scores + state + psi + weights


def implementation_extra_bytes_per_unit_step(w) -> dict:
    """What this implementation moves on top of that (streaming single-head path)."""
    e = 2 if w.dtype == "f16" else 4
    C, D, R, Rp = w.capacity, w.head_dim, w.rank, w.hidden
    nparts = (Rp + 63) // 64
    return {"fp64 accumulated scores (8 instead of 4 bytes, read and written)": 2 * 4 * C,
            "fp64 z (read and written)": 2 * 4 * R,
            "feature-map exchange array (written, read, handed back empty)": 3 * 2 * nparts * ((R + 3) // 4 * 4) * 4,
            "parked discarded pair: value row and psi (written, read next step), slot word": 2 * (D * e + 4 * R) + 8,
            "q and k rows read by the feature-map jobs as well": 2 * D * e,
            "token counter and eviction log": 12}


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
    ap.add_argument("--graph-reps", type=int, default=20, help="timed replays of the captured steps (at least 10)")
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

    unit_steps_per_s = U * args.steps / (ms * 1e-3)
    bytes_per_step = algorithmic_bytes_per_unit_step(w) * U
    achieved = bytes_per_step / (ms_per_step * 1e-3) / 1e9

    # The same steps as replays of a HIP graph (what a serving loop would run): one graph of
    # `graph_steps` steps, replayed `graph_reps` times, each replay timed by itself.
    graph_steps, graph_reps = 8 * L, max(10, args.graph_reps)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        run(0, L)                                          # first launches on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            run(0, graph_steps)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for _ in range(3):
        graph.replay()
    torch.cuda.synchronize()
    rep_ms = []
    for _ in range(graph_reps):
        e0.record(stream)
        graph.replay()
        e1.record(stream)
        torch.cuda.synchronize()
        rep_ms.append(e0.elapsed_time(e1) / graph_steps)
    rep_ms.sort()

    # The read rate this chip sustains for a stream shaped like the step's: the probe kernel over
    # a buffer as large as the cycled working set, one wave per region as in the step.
    from paper_2402_09398_amd import lessdec_probe_stream_read
    probe_bytes = 1 << 30
    pbuf = torch.empty((probe_bytes,), dtype=torch.uint8, device=dev).fill_(1)
    psink = torch.zeros((8192,), dtype=torch.int32, device=dev)
    for _ in range(3):
        lessdec_probe_stream_read(pbuf, probe_bytes, 8192, psink)
    torch.cuda.synchronize()
    e0.record(stream)
    for _ in range(10):
        lessdec_probe_stream_read(pbuf, probe_bytes, 8192, psink)
    e1.record(stream)
    torch.cuda.synchronize()
    probe_gbs = 10 * probe_bytes / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del pbuf

    from paper_2402_09398_amd.binding import lessdec_step_launches
    launches = lessdec_step_launches(layers[0].desc)
    one_launch = launches == 1
    extras = implementation_extra_bytes_per_unit_step(w) if w.q_per_kv == 1 else {}
    fp64_flops = U * G * (Pn ** 2 * D + 2.0 * min(Cn, Pn) * Pn * D * 0.5)    # row pass + exact columns of the kept/doubtful tokens (about)
    fp16_flops = prefill_flops - U * G * Pn ** 2 * D                          # everything else: A V, cheap column sums, psi, state
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
        # the whole step: on the headline workload one launch (feature-map jobs + attention waves)
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(w.cfg) if L >= 8 and w.q_per_kv == 1 and flags == 0 and one_launch else None,
                     "kernel": ("wpu_step_kernel" + (" (one launch per step: feature-map jobs and attention waves)"
                                                     if one_launch else " + mlp_parts_kernel (two launches per step)")
                                if w.q_per_kv == 1 else
                                ("gqs_step_kernel (one launch per step: feature-map jobs and a wave per query head)"
                                 if launches == 1 else f"grouped-head step kernel + feature-map kernel ({launches} launches per step)")),
                     "launches_per_step": launches,
                     "bytes_per_launch": bytes_per_step, "ms_per_launch": ms_per_step,
                     "algorithmic_bytes_per_unit_step": algorithmic_bytes_per_unit_step(w),
                     "implementation_extra_bytes_per_unit_step": extras,
                     "frac_with_extras": (bytes_per_step + sum(extras.values()) * U) / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "kv_only_frac": 2 * w.capacity * D * (2 if w.dtype == "f16" else 4) * U
                                     / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "stream_probe": {"GB/s": probe_gbs, "frac_of_probe": achieved / probe_gbs,
                                      "what": "lessdec_probe_stream_read: 1 GiB read once by 8192 waves, 7 KiB in flight each"},
                     "graph_replay": {"reps": graph_reps, "steps_per_replay": graph_steps,
                                      "ms_per_step_median": rep_ms[len(rep_ms) // 2], "ms_per_step_min": rep_ms[0],
                                      "frac_median": bytes_per_step / (rep_ms[len(rep_ms) // 2] * 1e-3) / 1e9 / HBM_PEAK_GBS}},
        # the prompt phase (secondary path), one warm call.  No per-kernel times are available inside
        # the process, so each class of matrix work is divided by the time of the WHOLE call: lower
        # bounds of what its kernels reach (per-kernel figures: profiles/).
        "prefill": {"ms": prefill_ms, "prompt_tokens_per_s": U * w.prompt / (prefill_ms * 1e-3),
                    "bound": "mfma",
                    "fp64_matrix": {"flops": fp64_flops, "achieved": fp64_flops / (prefill_ms * 1e-3) / 1e12, "peak": 78.6,
                                    "unit": "TFLOP/s", "frac": fp64_flops / (prefill_ms * 1e-3) / 1e12 / 78.6,
                                    "what": "Q K^T of the row pass and the exact column sums (they decide the heavy set)"},
                    "fp16_matrix": {"flops": fp16_flops, "achieved": fp16_flops / (prefill_ms * 1e-3) / 1e12, "peak": 2500.0,
                                    "unit": "TFLOP/s", "frac": fp16_flops / (prefill_ms * 1e-3) / 1e12 / 2500.0,
                                    "what": "A V, the cheap column sums, psi of the prompt keys, the state build"},
                    "note": "each class over the time of the whole call (a lower bound for its own kernels)"},
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, min(args.cpu_units, U), min(args.cpu_steps, T), flags)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
