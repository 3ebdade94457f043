#!/usr/bin/env python3
"""Benchmark: BPTT neuron-timesteps/s (forward + backward) of the LIF-SNN hot path on one MI355X.

One "step" = one whole training step over one synthetic batch that is already resident in HBM:
input-spike packing, event-driven forward with the strategy's state storage, loss, recomputation
from checkpoints, adjoint recurrence and weight-gradient accumulation (everything behind
snn_bind_inputs + snn_bptt).  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1] [--strategy remote]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth

# strategy parameters per benchmark configuration: (coarse, fine) and the HBM activation budget
STRATEGY_PARAMS = {
    0: {"standard": (0, 0), "chunk": (0, 10), "remote": (10, 0), "double": (20, 5)},
    1: {"standard": (0, 0), "chunk": (0, 32), "remote": (32, 0), "double": (100, 10)},
    2: {"standard": (0, 0), "chunk": (0, 100), "remote": (100, 0), "double": (100, 10)},
    3: {"standard": (0, 0), "chunk": (0, 316), "remote": (316, 0), "double": (316, 18)},
}
BUDGET = {2: 8 * 10**9, 3: 4 * 10**9}


def gather_bytes(w, rates, T, in_rate):
    """Algorithmic bytes of one forward (or recompute) pass: the weight rows of every active
    presynaptic spike (4*N_l bytes per event and target layer) plus the spike bits written/read."""
    total = 0.0
    pre_n, pre_r = w.n_in, in_rate
    for l, n in enumerate(w.n_hidden):
        ev_in = pre_r * pre_n * w.B * T
        ev_rec = rates[l] * n * w.B * T
        total += 4.0 * n * (ev_in + ev_rec) + (n / 8.0) * w.B * T
        pre_n, pre_r = n, rates[l]
    return total


def adjoint_bytes(w, T):
    """Dense transposed products: each matrix read once per step for the whole batch, plus the
    state read and the delta_v write (4+4 bytes per neuron, batch element and step)."""
    total = 0.0
    L = len(w.n_hidden)
    for l, n in enumerate(w.n_hidden):
        up = w.n_out if l == L - 1 else w.n_hidden[l + 1]
        total += 4.0 * n * (up + n) * T + 8.0 * n * w.B * T
    return total


def dw_bytes(w, rates, T, in_rate, launches):
    """delta_v row reads for every active presynaptic spike + one fp64 read-modify-write of every
    gradient matrix per launch."""
    total = 0.0
    pre_n, pre_r = w.n_in, in_rate
    for l, n in enumerate(w.n_hidden):
        total += 4.0 * n * (pre_r * pre_n + rates[l] * n) * w.B * T + 16.0 * (pre_n * n + n * n) * launches
        pre_n, pre_r = n, rates[l]
    total += 4.0 * w.n_out * rates[-1] * w.n_hidden[-1] * w.B * T + 16.0 * w.n_hidden[-1] * w.n_out * launches
    return total


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=1)
    ap.add_argument("--strategy", default="remote", choices=["standard", "chunk", "remote", "double"])
    ap.add_argument("--T", type=int, default=0, help="override the sequence length")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import synth
    import paper_2412_11810_amd as snn

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    w = synth.config(args.config, **({"T": args.T} if args.T else {}))
    d = synth.generate(w)
    dev = torch.device("cuda:0")
    x = torch.from_numpy(d["in_spikes"]).to(dev)
    y = torch.from_numpy(d["labels"]).to(dev)
    stream = torch.cuda.current_stream().cuda_stream
    net = snn.from_workload(w, d, stream=stream)
    sid = {"standard": snn.SNN_STANDARD, "chunk": snn.SNN_CHUNK, "remote": snn.SNN_REMOTE, "double": snn.SNN_DOUBLE}
    params = STRATEGY_PARAMS[args.config]
    budget = BUDGET.get(args.config, 0)

    def step(name, stats=False):
        C, F = params[name]
        net.snn_bind_inputs(x, y, w.T)
        return net.snn_bptt(sid[name], C, F, budget, want_stats=stats)

    def time_strategy(name, steps, warmup):
        for _ in range(warmup):
            step(name)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step(name)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    nts = w.neuron_timesteps()
    sec = time_strategy(args.strategy, args.steps, args.warmup)
    others = {}
    for name in params:
        if name != args.strategy:
            try:
                others[name] = nts / time_strategy(name, max(2, args.steps // 4), 1)
            except snn.SnnError as e:
                others[name] = str(e)

    # instrumented call of the timed strategy: per-kernel-kind durations from HIP events on the stream
    st = step(args.strategy, stats=True)
    rates = list(st.firing_rate)[: len(w.n_hidden)]
    in_rate = float(d["in_spikes"].mean())
    C, F = params[args.strategy]
    slots, rslots = snn.snn_state_slots(sid[args.strategy], w.T, C, F)
    n_bwd_launch = max(1, sum(1 for o in snn.snn_schedule(sid[args.strategy], w.T, C, F) if o[0] == "BACKWARD"))
    n_rec_launch = max(1, sum(1 for o in snn.snn_schedule(sid[args.strategy], w.T, C, F) if o[0] in ("REFWD1", "REFWD2")))
    n_fwd_launch = max(1, rslots)
    kinds = {
        "forward_gather": (st.ms_forward, gather_bytes(w, rates, w.T, in_rate), n_fwd_launch),
        "recompute_gather": (st.ms_recompute, gather_bytes(w, rates, st.refwd1_steps + st.refwd2_steps, in_rate), n_rec_launch),
        "adjoint": (st.ms_adjoint, adjoint_bytes(w, w.T), n_bwd_launch),
        "dw_scatter": (st.ms_dw, dw_bytes(w, rates, w.T, in_rate, n_bwd_launch), n_bwd_launch),
    }
    dom = max(kinds, key=lambda k: kinds[k][0])
    ms, byts, launches = kinds[dom]
    achieved = byts / (ms * 1e-3) / 1e9 if ms > 0 else 0.0
    roofline = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 5), "traffic": None,
                "launches_per_step": launches, "avg_launch_ms": round(ms / launches, 4),
                "algorithmic_bytes_per_launch": int(byts / launches),
                "per_kind": {k: {"ms_per_step": round(v[0], 3), "GB/s": round(v[1] / (v[0] * 1e-3) / 1e9, 2) if v[0] > 0 else None}
                             for k, v in kinds.items()}}

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "16")), w.B)
        Tcpu = min(w.T, 1000 if w.neurons <= 1024 else 100)
        t0 = time.perf_counter()
        oracle.bptt(w.n_in, list(w.n_hidden), w.n_out, d["W_in"], d["W_rec"], d["W_out"],
                    np.ascontiguousarray(d["in_spikes"][:Tcpu]), d["labels"], alpha=w.alpha, beta=w.beta,
                    theta=w.theta, surr_beta=w.surr_beta, dtype=np.float32, nthreads=cores)
        dt = time.perf_counter() - t0
        cpu = {"value": round(w.B * Tcpu * w.neurons / dt, 1), "unit": "neuron-timesteps/s", "cores": cores,
               "kind": "oracle", "sample": f"oracle fp32 Standard BPTT, first {Tcpu} of {w.T} steps, full batch, {dt:.2f} s wall"}

    out = {
        "metric": "BPTT neuron-timesteps/sec (fwd+bwd) at fixed HBM budget",
        "value": round(nts / sec, 1), "unit": "neuron-timesteps/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(sec * 1e3, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "T": w.T, "batch": w.B, "strategy": args.strategy, "coarse_interval": C,
                   "fine_interval": F, "hbm_budget_bytes": budget,
                   "hbm_activation_bytes": int(st.bytes_states + st.bytes_spikes + st.bytes_workspace),
                   "state_slots_hbm": slots, "state_slots_host": rslots,
                   "firing_rate": [round(r, 4) for r in rates], "input_rate": round(in_rate, 4),
                   "host_link_bytes_per_step": int(st.d2h_bytes + st.h2d_bytes),
                   "other_strategies_neuron_timesteps_per_s": {k: (round(v, 1) if not isinstance(v, str) else v) for k, v in others.items()}},
        "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(out))
    net.snn_destroy()


if __name__ == "__main__":
    main()
