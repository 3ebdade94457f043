#!/usr/bin/env python3
"""Benchmark: BPTT neuron-timesteps/s (forward + backward) of the LIF-SNN hot path on one MI355X.

One "step" = one whole training step over one synthetic batch that is already resident in HBM:
input-spike packing, event-driven forward with the strategy's state storage, loss, recomputation
from checkpoints, adjoint pass and weight-gradient accumulation (everything behind
snn_bind_inputs + snn_bptt).  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--strategy double]

The default workload is configuration 4 (1024 -> 4 x 8192 -> 100, T = 5000, batch 32, recurrent matrices 90 % zero),
the largest one of the benchmark configurations and the only one whose weights (1.9 GB) do not fit on the chip, run
with Double Checkpointing under its 32 GB HBM activation budget.

Other modes (used to produce the summaries under profiles/):
  --pmc-copy      run only the plain copy kernel (reference for scaling hardware byte counters)
  --single        one un-instrumented step of the chosen strategy and nothing else
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
_T0 = time.perf_counter()


def progress(msg):
    """Progress lines go to stderr (stdout carries the one JSON line): a step of the largest workload takes seconds."""
    print(f"[bench {time.perf_counter() - _T0:7.1f} s] {msg}", file=sys.stderr, flush=True)

HBM_PEAK_GBS = 8000.0     # MI355X published HBM3E bandwidth
MFMA_F32_PEAK_TF = 157.3  # MI355X published fp32 matrix peak
ALU_F32_PEAK_TF = 157.3   # MI355X published fp32 vector peak (256 CUs x 4 SIMDs x 64 flop/clk x 2.4 GHz)

# strategy parameters per benchmark configuration: (coarse, fine); budgets from the configurations
STRATEGY_PARAMS = {
    0: {"standard": (0, 0), "chunk": (0, 10), "remote": (10, 0), "double": (20, 5), "hier": (2, 10)},
    1: {"standard": (0, 0), "chunk": (0, 32), "remote": (32, 0), "double": (100, 10), "hier": (4, 32)},
    2: {"standard": (0, 0), "chunk": (0, 100), "remote": (100, 0), "double": (100, 10), "hier": (4, 100)},
    3: {"standard": (0, 0), "chunk": (0, 316), "remote": (316, 0), "double": (316, 18), "hier": (4, 316)},
    4: {"standard": (0, 0), "chunk": (0, 64), "remote": (64, 0), "double": (512, 64), "hier": (4, 64)},
}
BUDGET = {2: 8 * 10**9, 3: 4 * 10**9, 4: 32 * 10**9}
SID = {"standard": 0, "chunk": 1, "remote": 2, "double": 3, "hier": 4}  # hier: (nb_local, chunk)


def work_model(w, rates, in_rate, T, refwd_steps, rec_density, cur_steps=None, dw_tile_chunks=0, csr_recompute=False):
    """Own work of one training step per kernel kind: what the event-driven method must do, whatever a kernel
    does internally -- bytes of the weight rows of ACTIVE presynaptic neurons (existing synapses only for a masked
    recurrent matrix kept as compressed rows: 4-byte value + 2-byte index), one add per such weight, the dense
    recurrent product of the adjoint pass (dense by necessity: the surrogate derivative has no compact support)
    and the dense inter-layer products.  Event counts come from the measured firing rates."""
    B, L = w.B, len(w.n_hidden)
    N = w.n_hidden
    pre_n = [w.n_in] + list(N[:-1])
    pre_r = [in_rate] + list(rates[:-1])
    ev_in = [pre_r[l] * pre_n[l] * B for l in range(L)]       # feed-forward events per step (whole batch)
    ev_rec = [rates[l] * N[l] * B for l in range(L)]          # recurrent events per step
    ev_out = rates[-1] * N[-1] * B
    masked = rec_density < 1.0
    # bytes of one recurrent row: the method's own figure for a masked matrix is a weight and a 16-bit index per existing
    # synapse (6 bytes); the gather and adjoint kernels read a packed 8-byte entry, which the counters show, not this model
    row_rec = [(6.0 * rec_density if masked else 4.0) * N[l] for l in range(L)]
    ent_rec = [(rec_density if masked else 1.0) * N[l] for l in range(L)]         # weights in one recurrent row
    out = {}
    out["fwd_currents"] = ("hbm", T * (sum(4.0 * N[l] * ev_in[l] + 8.0 * N[l] * B for l in range(L)) + 4.0 * w.n_out * ev_out))
    seq_adds = T * sum(ent_rec[l] * ev_rec[l] for l in range(L) if N[l] <= 256)
    seq_bytes = T * sum(row_rec[l] * ev_rec[l] + (N[l] / 8.0 + 4.0 * N[l]) * B for l in range(L) if N[l] > 256)
    out["fwd_seq"] = ("alu", seq_adds) if max(N) <= 256 else ("hbm", seq_bytes)
    # recompute: part 1, the currents (weight rows of the events + the current written) and part 2, the scan (current
    # read, state written, one spike bit read)
    # (cur_steps: the steps whose currents the recompute passes actually computed -- Double keeps a segment's currents
    # between its two passes when the budget has room, so they are computed once)
    cur_steps = refwd_steps if cur_steps is None else cur_steps
    out["recompute"] = ("hbm", cur_steps * sum(4.0 * N[l] * ev_in[l] + row_rec[l] * ev_rec[l] + 4.0 * N[l] * B for l in range(L)))
    out["scan"] = ("hbm", refwd_steps * sum((8.0 + 1.0 / 8.0) * N[l] * B for l in range(L)))
    # adjoint recurrence: layers wider than 1024 stream their recurrent matrix once per step for the whole batch
    if max(N) > 1024:
        out["adjoint"] = ("hbm", T * sum((6.0 * rec_density if masked else 4.0) * N[l] * N[l] for l in range(L) if N[l] > 1024))
    else:
        out["adjoint"] = ("alu", sum(2.0 * ent_rec[l] * N[l] * B * T for l in range(L)))
    up = [w.n_out if l == L - 1 else N[l + 1] for l in range(L)]
    out["up_gemm"] = ("mfma32", sum(2.0 * N[l] * up[l] * B * T for l in range(L)))
    # weight gradients: read-modify-write of the gradient rows of active presynaptic neurons (fp32 in, fp32 out)
    dw_bytes = T * (sum(8.0 * N[l] * ev_in[l] + 8.0 * ent_rec[l] * ev_rec[l] for l in range(L)) + 8.0 * w.n_out * ev_out)
    dw_adds = T * (sum(N[l] * ev_in[l] + ent_rec[l] * ev_rec[l] for l in range(L)) + w.n_out * ev_out)
    out["dw"] = ("hbm", dw_bytes)
    if dw_tile_chunks:
        # the tiled event-driven kernel keeps the fp64 accumulators of a tile in registers for a whole launch (one
        # adjoint tile of the backward pass): its own HBM work is the accumulators read and written once per launch,
        # the adjoint rows of every matrix's postsynaptic layer read once and the spike words -- far below the
        # read-modify-write per event of the scatter form priced above
        # (a masked recurrent matrix keeps one accumulator per existing synapse when batch <= 32)
        rec_frac = rec_density if (masked and B <= 32 and os.environ.get("SNN_DW_CSR", "") != "0" and os.environ.get("SNN_CSR", "") != "0") else 1.0
        entries = sum(pre_n[l] * N[l] + rec_frac * N[l] * N[l] for l in range(L)) + N[-1] * w.n_out
        rows = T * B * (sum(4.0 * 2 * N[l] + (pre_n[l] + N[l]) / 8.0 for l in range(L)) + 4.0 * w.n_out + N[-1] / 8.0)
        out["dw"] = ("hbm", dw_tile_chunks * 16.0 * entries + rows)
    # fused launches of the narrow-layer networks: the recurrences (dense) + the adds of the weight gradients and of
    # the recompute currents that ride along; the forward stage: the adds of the active rows
    rec_adds = cur_steps * sum(N[l] * ev_in[l] + ent_rec[l] * ev_rec[l] for l in range(L))
    out["bwd_stage"] = ("alu", sum(2.0 * N[l] * N[l] * B * T for l in range(L)) + dw_adds + rec_adds)
    out["fwd_stage"] = ("alu", T * sum(N[l] * ev_in[l] + ent_rec[l] * ev_rec[l] for l in range(L)))
    out["bwd_inter"] = out["up_gemm"]
    # what the dense matrix-core current kernel (matrices far beyond the L2) actually executes: one K = 1 matrix
    # operation per presynaptic neuron whether it spiked or not -- its own bound, reported beside the own-work figure
    # (which it can exceed: a weight row streamed once serves 64 (t, b) rows)
    dense = {"fwd_currents": 2.0 * B * T * (sum(pre_n[l] * N[l] for l in range(L)) + N[-1] * w.n_out)}
    dense["recompute"] = 2.0 * B * cur_steps * sum(pre_n[l] * N[l] + (0 if csr_recompute else N[l] * N[l]) for l in range(L))
    # the matrix-core contraction of the weight gradients (k_dw_mfma): spikes as 0/1 operands, every (t, b) row
    dense["dw"] = 2.0 * B * T * (sum(pre_n[l] * N[l] + N[l] * N[l] for l in range(L)) + N[-1] * w.n_out)
    # the list version of the currents (k_currents_mfma): one K = 1 operation per presynaptic neuron that is active in
    # a block of 16 (t, b) rows -- the union over 16 rows of independent spikes at rate r is 1 - (1 - r)^16
    un = lambda r: 1.0 - (1.0 - min(max(r, 0.0), 1.0)) ** 16
    lst_fw = 2.0 * B * T * (sum(un(pre_r[l]) * pre_n[l] * N[l] for l in range(L)) + un(rates[-1]) * N[-1] * w.n_out)
    lst_re = 2.0 * B * cur_steps * sum((un(pre_r[l]) * pre_n[l] + un(rates[l]) * N[l]) * N[l] for l in range(L))
    out["_list_flops"] = {"fwd_currents": lst_fw, "recompute": lst_re}
    out["_dense_flops"] = dense
    return out


def read_traffic(workload, strategy, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary, or None."""
    path = os.path.join(ROOT, "profiles", f"pmc_traffic_{workload}_{strategy}.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        p = line.split()
        if len(p) >= 4 and p[0] == "kernel" and p[1] == kernel.replace(" ", ""):
            kv = dict(zip(p[2::2], p[3::2]))
            try:
                return float(kv["fetch_bytes_per_launch"]) + float(kv["write_bytes_per_launch"])
            except (KeyError, ValueError):
                return None
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4)
    ap.add_argument("--strategy", default="double", choices=list(SID))
    ap.add_argument("--T", type=int, default=0, help="override the sequence length")
    ap.add_argument("--gain", type=float, default=0.0, help="override the weight gain (sets the hidden firing rate)")
    ap.add_argument("--coarse", type=int, default=-1)
    ap.add_argument("--fine", type=int, default=-1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--others", default="auto", choices=["auto", "all", "none"],
                    help="time the other strategies too (auto: all of them for configurations 0 and 1, none otherwise)")
    ap.add_argument("--no-long", action="store_true", help="skip the 10x-sequence-length comparison")
    ap.add_argument("--no-tight", action="store_true",
                    help="skip the same strategy under the smallest budget it can run in (snn_bytes_required)")
    ap.add_argument("--long-reps", type=int, default=1)
    ap.add_argument("--budget", type=int, default=-1, help="HBM activation budget in bytes (default: the configuration's)")
    ap.add_argument("--single", action="store_true")
    ap.add_argument("--sweep", action="store_true", help="chunk-size / remote-chunk-size study (use with --T 4096)")
    ap.add_argument("--host-inputs", action="store_true",
                    help="hand the input spikes over as host arrays every step (PCIe-inclusive rate; not the headline value)")
    ap.add_argument("--pmc-copy", action="store_true")
    ap.add_argument("--micro-currents", action="store_true",
                    help="current kernels alone on teacher-forced hidden spike trains at 1 / 5 / 20 %% (use with --config, --T, --fine)")
    ap.add_argument("--model-sweep", action="store_true",
                    help="largest hidden width per strategy at fixed T and HBM budget (use with --T and --budget-mb)")
    ap.add_argument("--budget-mb", type=float, default=200.0)
    ap.add_argument("--spike-tier", type=int, default=0, choices=[0, 1],
                    help="1: the hidden layers' spike bitmasks of finished coarse segments live in pinned host memory (Remote / Double)")
    ap.add_argument("--surr-window", type=float, default=0.0,
                    help="surrogate window w (not in the paper): derivative cut to 0 where |v - theta| >= w; <= 0: none")
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
    dev = torch.device("cuda:0")

    if args.pmc_copy:
        net = snn.Snn(snn.make_config(8, [64], 2, 4, 1))
        nbytes = 256 << 20
        a = torch.ones(nbytes // 4, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        for _ in range(3):
            net.snn_debug_copy(a, b, nbytes)
        print(json.dumps({"copy_bytes_read": nbytes, "copy_bytes_written": nbytes, "launches": 3}))
        return

    if args.model_sweep:
        # Model-size scaling (the shape of the paper's Fig. 2 right / Fig. 3): at a fixed sequence length and HBM
        # activation budget, the widest two-layer network (700 -> N -> N -> 20, batch 32, widths in steps of 64)
        # each strategy can train -- closed form from snn_bytes_required, intervals by the square-root rules --
        # and one training step actually run at that width (Standard's and Double's).
        T = args.T or 4096
        budget_b = int(args.budget_mb * 1e6)
        rows = []
        for name in ("standard", "chunk", "remote", "double", "hier"):
            sid = SID[name]
            lo, hi = 0, 8192 // 64
            while lo < hi:  # largest N = 64*k with bytes_required <= budget
                mid = (lo + hi + 1) // 2
                need = snn.snn_bytes_required(snn.make_config(700, [64 * mid] * 2, 20, T, 32), sid, T, 0, 0)
                if 0 < need <= budget_b:
                    lo = mid
                else:
                    hi = mid - 1
            N = 64 * lo
            row = {"strategy": name, "max_width": N, "neurons": 2 * N}
            if N >= 64:
                cfgN = snn.make_config(700, [N] * 2, 20, T, 32)
                row["bytes_required"] = snn.snn_bytes_required(cfgN, sid, T, 0, 0)
                row["state_slots_hbm"], row["state_slots_host"] = snn.snn_state_slots(sid, T, 0, 0)
                if name in ("standard", "double"):
                    wl = synth.Workload(f"model_sweep_700-2x{N}-20", 700, (N, N), 20, T=T, B=32, p_in=0.02,
                                        gain=1.0 if N <= 256 else 0.2, seed=1)
                    dd = synth.generate(wl)
                    nn_ = snn.from_workload(wl, dd)
                    xx = torch.from_numpy(dd["in_spikes"]).to(dev)
                    yy = torch.from_numpy(dd["labels"]).to(dev)
                    nn_.snn_bind_inputs(xx, yy, T)
                    nn_.snn_bptt(sid, 0, 0, budget_b, want_stats=False)
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                    nn_.snn_bind_inputs(xx, yy, T)
                    nn_.snn_bptt(sid, 0, 0, budget_b, want_stats=False)
                    torch.cuda.synchronize()
                    row["ms_per_step"] = round((time.perf_counter() - t0) * 1e3, 2)
                    row["neuron_timesteps_per_s"] = round(32 * T * 2 * N / (time.perf_counter() - t0), 1)
                    nn_.snn_destroy()
            rows.append(row)
        print(json.dumps({"model_sweep": "700->N->N->20, batch 32", "T": T, "budget_bytes": budget_b, "rows": rows}))
        return

    w = synth.config(args.config, **({"T": args.T} if args.T else {}), **({"gain": args.gain} if args.gain else {}))
    progress(f"drawing the synthetic workload {w.name} (T={w.T}, batch {w.B})")
    d = synth.generate(w)
    progress("workload drawn; loading weights")
    x = torch.from_numpy(d["in_spikes"]).to(dev)
    y = torch.from_numpy(d["labels"]).to(dev)
    if args.host_inputs:  # the library copies them to the device inside snn_bind_inputs, every step
        x, y = d["in_spikes"], d["labels"]
    net = snn.from_workload(w, d, surr_window=args.surr_window, spike_tier=args.spike_tier)  # stream = None: the library runs on a stream of its own
    params = dict(STRATEGY_PARAMS[args.config])
    if args.coarse >= 0 or args.fine >= 0:
        c0, f0 = params[args.strategy]
        params[args.strategy] = (args.coarse if args.coarse >= 0 else c0, args.fine if args.fine >= 0 else f0)
    for name, (c_, f_) in list(params.items()):  # a shortened sequence (--T) shortens the intervals with it
        if name == "hier":
            params[name] = (c_, min(f_, w.T))
        else:
            c2 = min(c_, w.T) if c_ else 0
            params[name] = (c2, min(f_, c2 if c2 else w.T) if f_ else 0)
    budget = args.budget if args.budget >= 0 else BUDGET.get(args.config, 0)
    if args.config in (0, 1) and args.budget < 0:
        # configurations 0 and 1 name no budget: every strategy runs inside what plain BPTT needs for this T
        budget = snn.snn_bytes_required(snn.make_config(w.n_in, list(w.n_hidden), w.n_out, w.T, w.B), snn.SNN_STANDARD, w.T)

    def step(name, stats=False):
        C, F = params[name]
        net.snn_bind_inputs(x, y, w.T)
        return net.snn_bptt(SID[name], C, F, budget, want_stats=stats)

    if args.micro_currents:
        # Kernel micro-benchmark at a controlled activity level: hidden spike trains drawn i.i.d. at an exact rate
        # (decoupled from the dynamics) replace the stored ones, and the synaptic-current part of recompute runs
        # over the whole sequence in chunks of --fine steps, with each of the three kernels.  "event_row_GBs" is the
        # event-driven method's own traffic (one weight row of 4 N_l bytes per presynaptic spike) over the time.
        net.snn_bind_inputs(x, y, w.T)
        L = len(w.n_hidden)
        chunk = args.fine if args.fine >= 1 else 10
        in_rate = float(d["in_spikes"].mean())
        pre_n = [w.n_in] + list(w.n_hidden[:-1])
        rows = []
        for rate in (0.01, 0.05, 0.2):
            hid = [torch.from_numpy(h).to(dev) for h in synth.forced_spike_trains(w, [rate] * L)]
            ev_bytes = w.T * w.B * sum(4.0 * w.n_hidden[l] * ((in_rate if l == 0 else rate) * pre_n[l] + rate * w.n_hidden[l])
                                       for l in range(L))
            dense_flops = w.T * w.B * sum(2.0 * w.n_hidden[l] * (pre_n[l] + w.n_hidden[l]) for l in range(L))
            # own bytes when the recurrent rows are compressed (6 bytes per existing synapse)
            ev_bytes_csr = w.T * w.B * sum(w.n_hidden[l] * (4.0 * (in_rate if l == 0 else rate) * pre_n[l] + 6.0 * w.rec_density * rate * w.n_hidden[l])
                                           for l in range(L))
            modes = [("gather", "0"), ("mfma", "0"), ("dense", "0")]
            if w.rec_density < 1.0:  # masked recurrent matrices: the recurrent part over compressed rows
                modes += [("gather", "1"), ("dense", "1")]
            for mode, csr in modes:
                os.environ["SNN_CURRENTS"] = mode
                os.environ["SNN_CSR"] = csr
                ms = net.snn_debug_currents(hid, chunk, reps=2)
                name = {"gather": "k_currents", "mfma": "k_currents_mfma", "dense": "k_currents_dense"}[mode]
                rows.append({"rate": rate, "kernel": name + (" (feed-forward) + k_currents_csr (recurrent)" if csr == "1" else ""),
                             "ms_per_pass": round(ms, 3), "event_row_GBs": round((ev_bytes_csr if csr == "1" else ev_bytes) / ms / 1e6, 1),
                             "dense_TFLOPs": round(dense_flops / ms / 1e9, 2)})
            del hid
        os.environ.pop("SNN_CURRENTS", None)
        os.environ.pop("SNN_CSR", None)
        print(json.dumps({"micro_currents": w.name, "T": w.T, "batch": w.B, "chunk": chunk, "input_rate": round(in_rate, 4), "rows": rows}))
        net.snn_destroy()
        return

    if args.sweep:
        # Hyper-parameter study (shape of the paper's Figs. 4-5): time per step and HBM state memory
        # against the chunk size (Chunk, Remote), the number of checkpoints per transfer (Hier) and the
        # remote chunk size with chunk = sqrt(remote chunk) (Double).
        Ms = 4 * w.B * w.neurons
        rows = []

        def run(name, sid, C, F, reps=3):
            net.snn_bind_inputs(x, y, w.T)
            net.snn_bptt(sid, C, F, 0, want_stats=False)
            net.snn_bptt(sid, C, F, 0, want_stats=False)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                net.snn_bind_inputs(x, y, w.T)
                net.snn_bptt(sid, C, F, 0, want_stats=False)
            torch.cuda.synchronize()
            slots, rs = snn.snn_state_slots(sid, w.T, C, F)
            rows.append({"strategy": name, "coarse": C, "fine": F, "ms_per_step": round((time.perf_counter() - t0) / reps * 1e3, 3),
                         "state_slots_hbm": slots, "state_bytes_hbm": slots * Ms, "state_slots_host": rs})
        run("standard", snn.SNN_STANDARD, 0, 0)
        for F in (8, 16, 32, 64, 128, 256, 512):
            run("chunk", snn.SNN_CHUNK, 0, F)
        for Cc in (8, 16, 32, 64, 128, 256, 512):
            run("remote", snn.SNN_REMOTE, Cc, 0)
        for NL in (1, 2, 4, 8, 16):
            run("hier", snn.SNN_HIER, NL, 64)
        for Cc in (16, 64, 256, 1024, 4096):
            run("double", snn.SNN_DOUBLE, Cc, max(1, int(round(Cc ** 0.5))))
        for Ff in (2, 4, 8, 16, 32, 64):
            run("double", snn.SNN_DOUBLE, 256, Ff)
        print(json.dumps({"sweep": w.name, "T": w.T, "batch": w.B, "M_s_bytes": Ms, "rows": rows}))
        net.snn_destroy()
        return

    if args.single:
        step(args.strategy)
        torch.cuda.synchronize()
        print(json.dumps({"single_step": args.strategy, "workload": w.name}))
        net.snn_destroy()
        return

    def time_strategy(name, steps, warmup):
        for i in range(warmup):
            step(name)
            progress(f"{name}: warm-up step {i + 1}/{warmup} done")
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        last = t0
        for i in range(steps):
            step(name)
            if time.perf_counter() - last > 20.0:  # (each call returns after its step has completed)
                progress(f"{name}: timed step {i + 1}/{steps} done")
                last = time.perf_counter()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    nts = w.neuron_timesteps()
    sec = time_strategy(args.strategy, args.steps, args.warmup)
    others = {}
    if args.others == "all" or (args.others == "auto" and args.config in (0, 1)):
        for name in params:
            if name != args.strategy:
                try:
                    others[name] = round(nts / time_strategy(name, max(2, args.steps // 4), 2), 1)
                except snn.SnnError as e:
                    others[name] = str(e)

    # the same strategy and intervals under the smallest budget they can run in: no currents cache (Double recomputes
    # the currents twice), no buffers to pipeline the layers of the adjoint pass -- the other end of the trade
    tight = None
    if not args.no_tight and budget:
        Ct, Ft = params[args.strategy]
        need_min = int(snn.snn_bytes_required(net.cfg, SID[args.strategy], w.T, Ct, Ft))
        if 0 < need_min < budget:
            def step_tight():
                net.snn_bind_inputs(x, y, w.T)
                return net.snn_bptt(SID[args.strategy], Ct, Ft, need_min, want_stats=False)
            step_tight()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(2):
                step_tight()
            torch.cuda.synchronize()
            sec_t = (time.perf_counter() - t0) / 2
            tight = {"hbm_budget_bytes": need_min, "ms_per_step": round(sec_t * 1e3, 3), "neuron_timesteps_per_s": round(nts / sec_t, 1)}
            progress(f"under the smallest budget ({need_min} B): {sec_t * 1e3:.1f} ms per step")
            step(args.strategy)  # back to the timed plan (its graph is recorded again) before the instrumented steps

    # instrumented (eager) steps of the timed strategy: per-kernel-kind durations from HIP events
    # recorded on the stream the kernels run on; the second one is used (the first pays one-time costs)
    progress(f"timed: {sec * 1e3:.1f} ms per step; instrumented steps")
    step(args.strategy, stats=True)
    st = step(args.strategy, stats=True)
    progress("instrumented steps done")
    rates = list(st.firing_rate)[: len(w.n_hidden)]
    in_rate = float(d["in_spikes"].mean())
    C, F = params[args.strategy]
    slots, rslots = snn.snn_state_slots(SID[args.strategy], w.T, C, F)
    sched = snn.snn_schedule(SID[args.strategy], w.T, C, F)
    n_bwd = max(1, sum(-(-(o[1] - o[2] + 1) // 256) for o in sched if o[0] == "BACKWARD"))  # adjoint tiles of <= 256 steps
    Ms = 4 * w.B * w.neurons
    tier = os.environ.get("SNN_HOST_TIER", "")
    host_direct = args.strategy in ("remote", "double") and tier != "dma" and (tier == "direct" or Ms <= (1 << 20))
    seg = C if (args.strategy in ("remote", "double") and not host_direct) else (F if args.strategy == "hier" else w.T)
    n_tiles = sum(-(-(min(a + seg, w.T) - a) // 64) for a in range(0, w.T, seg))   # forward tiles of <= 64 steps
    n_rec = sum(1 for o in sched if o[0] == "REFWD2") + sum(-(-(o[2] - o[1]) // max(F, 1)) for o in sched if o[0] == "REFWD1")
    L = len(w.n_hidden)
    big = any(4.0 * max(pn, n) * n >= (32 << 20) for pn, n in zip([w.n_in] + list(w.n_hidden[:-1]), w.n_hidden))
    dw_env = os.environ.get("SNN_DW", "")
    # (the library's rule: always for matrices of 32 MB and more; for other networks with layers wider than 256 below
    # 8 % presynaptic activity averaged over the weight rows, from the second training step on)
    pre_rates = [in_rate] + list(rates[:-1])
    act = (sum((pre_rates[l] * (w.n_in if l == 0 else w.n_hidden[l - 1]) + rates[l] * w.n_hidden[l]) * w.n_hidden[l] for l in range(L)) /
           sum(((w.n_in if l == 0 else w.n_hidden[l - 1]) + w.n_hidden[l]) * w.n_hidden[l] for l in range(L)))
    dw_tile = w.B <= 64 and (dw_env == "tile" or (dw_env not in ("mfma", "event") and (big or (max(w.n_hidden) > 256 and act < 0.08))))
    model = work_model(w, rates, in_rate, w.T, st.refwd1_steps + st.refwd2_steps, w.rec_density,
                       cur_steps=st.refwd_current_steps or (st.refwd1_steps + st.refwd2_steps),
                       dw_tile_chunks=n_bwd if dw_tile else 0,
                       csr_recompute=big and w.rec_density < 1.0 and os.environ.get("SNN_CSR", "") != "0" and
                       (os.environ.get("SNN_CSR", "") == "1" or max(rates) * w.rec_density < 0.01))
    dense_flops = model.pop("_dense_flops")
    list_flops = model.pop("_list_flops")
    ms = {"fwd_seq": st.ms_fwd_seq, "fwd_currents": st.ms_fwd_currents, "recompute": st.ms_recompute, "scan": st.ms_scan,
          "adjoint": st.ms_adjoint, "up_gemm": st.ms_up_gemm, "dw": st.ms_dw, "bwd_stage": st.ms_bwd_stage,
          "fwd_stage": st.ms_fwd_stage, "bwd_inter": 0.0}
    # adjoint recurrence of layers wider than 1024: event-driven rows under a surrogate window, chip-wide over the
    # compressed rows for a masked matrix (all layers of a pipeline stage in one launch), else chip-wide over the
    # dense-stored matrix (one launch per layer and tile)
    ws_env = os.environ.get("SNN_WS_KERNEL", "")
    adj_kernel = ("k_adj_rec_rows" if (args.surr_window > 0 and ws_env in ("", "rows", "rows_all")) or ws_env in ("rows", "rows_all") else
                  "k_adj_rec_csrw" if (w.rec_density < 1.0 and w.B <= 64 and os.environ.get("SNN_CSR", "") != "0" and ws_env in ("", "csrw")) else
                  "k_adj_rec_wide")
    # inter-layer products of matrices from 2048 x 2048: one launch of the 128 x 128-tile kernel per product
    gemm_big = L > 1 and min(w.n_hidden) >= 2048
    # launches of each kind's main kernel per step (layers that share a width and a pipeline stage share a launch)
    n_stage = n_tiles + 2 * (L - 1)
    n_cur = n_rec
    if 0 < st.refwd_current_steps < st.refwd1_steps + st.refwd2_steps:
        # Double kept the currents of a coarse segment: one current launch per segment with a Re-Forward_1 pass, plus
        # one per chunk of the segments that have none
        cached = {o[1] // C for o in sched if o[0] == "REFWD1"}
        n_cur = len(cached) + sum(1 for o in sched if o[0] == "REFWD2" and o[1] // C not in cached)
    launches = {"fwd_seq": n_stage, "fwd_currents": n_stage, "recompute": max(1, n_cur), "scan": max(1, n_rec),
                "adjoint": n_bwd * L if (max(w.n_hidden) > 1024 and adj_kernel == "k_adj_rec_wide") else n_bwd + L - 1,
                "up_gemm": n_bwd * (L - 1) if gemm_big else max(1, n_bwd + L - 2),
                "dw": n_bwd + L - 1, "bwd_stage": max(1, n_bwd + L - 1),
                "fwd_stage": max(1, n_tiles + 2 * L - 2), "bwd_inter": max(1, n_bwd + L - 2)}
    if st.ms_bwd_stage > 0:
        # all but the first stage's recurrences and the last stage's weight gradients ran inside fused launches:
        # what is left of the two separate kinds is one launch each, not worth a line.  The launch between two
        # stages carries the inter-layer products and the recompute of the next two chunks (timed as one kind).
        ms["adjoint"] = ms["dw"] = 0.0
        ms["bwd_inter"], ms["up_gemm"] = ms["up_gemm"], 0.0
        if ms["recompute"] < 0.25 * ms["bwd_inter"]:  # only the first chunk's recompute ran on its own
            ms["recompute"] = 0.0
    fwd_fused_wide = False
    if st.ms_fwd_stage > 0:
        if big:
            # wide layers over compressed rows: the dense feed-forward currents for the next stage ride in the launch
            # of a stage's sequential parts (k_fwd_stage_csr); the few current launches that stay on their own (first
            # stage, readout) are counted with them
            fwd_fused_wide = True
            ms["fwd_stage"] += ms["fwd_seq"] + ms["fwd_currents"]
            model["fwd_stage"] = ("hbm", model["fwd_seq"][1] + model["fwd_currents"][1])  # own work: both kinds' row bytes
        ms["fwd_seq"] = ms["fwd_currents"] = 0.0
    wide = max(w.n_hidden) > 256
    # compressed rows of masked recurrent matrices: forced by SNN_CSR=1, else the library's policy (matrices of 32 MB and
    # more, firing rate x density below 0.01 in every layer)
    csr_env = os.environ.get("SNN_CSR", "")
    csr_pol = big and w.rec_density < 1.0 and max(rates) * w.rec_density < 0.01 and np.mean(rates) >= 0.035
    csr_fwd = w.rec_density < 1.0 and all(n % 2048 == 0 for n in w.n_hidden) and (csr_env == "1" or (csr_env == "" and (csr_pol or (big and np.mean(rates) < 0.035))))
    kernel_of = {"fwd_seq": ("k_layer_seq_gather" if os.environ.get("SNN_SEQ_KERNEL", "") == "gather" else "k_layer_seq_rs") if not wide else ("k_layer_seq_csr_sl" if csr_fwd else
                            ("k_layer_seq_gather_sl" if max(w.n_hidden) >= 2048 and max(w.n_hidden) % 1024 == 0 else "k_layer_seq_gather")),
                 # (matrices of 32 MB and more: the dense matrix-core version from 3.5 % presynaptic activity, below it
                 # the event-by-event gather k_currents, with k_currents_csr for masked recurrent matrices)
                 "fwd_currents": ("k_currents_dense<4,0>" if np.mean(rates) >= 0.035 else "k_currents") if big else "k_currents_mfma",
                 "recompute": ("k_currents_dense<4,1>" if np.mean(rates) >= 0.035 else "k_currents") if big else "k_currents_mfma",
                 "scan": "k_scan", "up_gemm": "k_up_gemm<4,4,2,2>" if gemm_big else ("k_bwd_inter" if L > 2 else "k_up_gemm"), "dw": "k_dw_tile" if dw_tile else "k_dw_mfma", "bwd_stage": "k_bwd_stage", "fwd_stage": "k_fwd_stage_csr" if fwd_fused_wide else "k_fwd_stage",
                 "bwd_inter": "k_bwd_inter",
                 "adjoint": "k_adj_rec_rs" if not wide else ("k_adj_rec_wsm" if max(w.n_hidden) <= 1024 else adj_kernel)}
    peaks = {"hbm": (HBM_PEAK_GBS, "GB/s", 1e9), "alu": (ALU_F32_PEAK_TF, "TFLOP/s", 1e12), "mfma32": (MFMA_F32_PEAK_TF, "TFLOP/s", 1e12)}
    kinds = {}
    for k, (bound, work) in model.items():
        if ms[k] <= 0:
            continue
        peak, unit, scale = peaks[bound]
        ach = work / (ms[k] * 1e-3) / scale
        kinds[k] = {"kernel": kernel_of[k], "bound": "mfma" if bound == "mfma32" else bound, "ms_per_step": round(ms[k], 3),
                    "launches_per_step": launches[k], "avg_launch_ms": round(ms[k] / launches[k], 4),
                    "achieved": round(ach, 3), "peak": round(peak, 1), "unit": unit, "frac": round(ach / peak, 5)}
        tr = read_traffic(w.name, args.strategy, kernel_of[k])
        if tr is not None:
            # HBM bytes per launch of this kernel from the committed counter summary (same launch shape; the recompute
            # launch there covers a shorter coarse segment, see the file's header) next to the own-work bytes per launch
            kinds[k]["traffic_bytes_per_launch"] = int(tr)
            if bound == "hbm":
                kinds[k]["own_bytes_per_launch"] = int(work / launches[k])
        what = None
        if k == "fwd_stage" and fwd_fused_wide:
            what, fl = ("dense K=1 fp32 matrix operations of the feed-forward currents, one per presynaptic neuron; the "
                        "sequential chain over compressed rows runs beside them in the same launch"), dense_flops["fwd_currents"]
        elif kernel_of[k].startswith("k_currents_dense") and k in dense_flops:
            what, fl = "dense K=1 fp32 matrix operations, one per presynaptic neuron", dense_flops[k]
        elif kernel_of[k] == "k_dw_mfma" and k == "dw":
            what, fl = "fp32 matrix operations over every (t, b) row, spikes as 0/1 operands", dense_flops[k]
        elif kernel_of[k] == "k_currents_mfma" and k in list_flops:
            what, fl = "K=1 fp32 matrix operations, one per presynaptic neuron active in a block of 16 rows (expected union)", list_flops[k]
        if what:
            # A matrix-core kernel is bound by the operations it executes, and it can exceed the event-driven method's
            # byte figure (a weight row fetched once serves every (t, b) row of its tile): the kind's bound is the
            # matrix peak, the own-work figure stays beside it.  (The recompute kind's time includes the gather over
            # compressed rows that serves its recurrent part, so its fraction is a lower bound for the dense kernel.)
            tf = fl / (ms[k] * 1e-3) / 1e12
            own = {f: kinds[k][f] for f in ("bound", "achieved", "peak", "unit", "frac")}
            kinds[k].update({"bound": "mfma", "achieved": round(tf, 3), "peak": MFMA_F32_PEAK_TF, "unit": "TFLOP/s",
                             "frac": round(tf / MFMA_F32_PEAK_TF, 5), "what": what, "own_work": own})
            model[k] = ("mfma32", fl)
    dom = max(kinds, key=lambda k: kinds[k]["ms_per_step"])
    dk = kinds[dom]
    work_per_launch = model[dom][1] / launches[dom]
    traffic = read_traffic(w.name, args.strategy, dk["kernel"])
    roofline = {"bound": dk["bound"], "kernel": dk["kernel"], "kind": dom, "achieved": dk["achieved"], "peak": dk["peak"],
                "unit": dk["unit"], "frac": dk["frac"], "traffic": traffic,
                "launches_per_step": dk["launches_per_step"], "avg_launch_ms": dk["avg_launch_ms"],
                "algorithmic_work_per_launch": int(work_per_launch),
                "note": "work = the event-driven method's own work per kind (bytes of the weight rows of active presynaptic "
                        "neurons -- existing synapses only for masked matrices -- for hbm kinds; adds of those rows plus the "
                        "dense recurrent product of the adjoint for alu kinds; dense inter-layer products for mfma kinds), "
                        "never the dense-equivalent work of a kernel; durations from HIP events on the compute stream of an "
                        "eager step; traffic = HBM bytes per launch of that kernel (FETCH_SIZE + WRITE_SIZE, scaled by the "
                        "copy kernel) from the committed rocprofv3 --pmc summary of this workload at the same launch shape "
                        "(profiles/pmc_traffic_<workload>_<strategy>.txt; null if none)",
                "kinds": kinds}

    # ---- measured peaks next to the published ones: a plain streaming copy (1 GiB read + 1 GiB written per
    # launch, the library's copy kernel) and pinned-host copies of one state (and of 64 MiB) in both directions ----
    def measured_peaks():
        n = 1 << 30
        a = torch.ones(n // 4, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        net.snn_debug_copy(a, b, n)
        t0 = time.perf_counter()
        for _ in range(5):
            net.snn_debug_copy(a, b, n)
        hbm = 5 * 2 * n / (time.perf_counter() - t0) / 1e9
        del a, b
        out = {"hbm_copy_GBs": round(hbm, 1)}
        for tag, m in (("", 64 << 20), ("_one_state", max(4096, Ms))):
            h = torch.empty(m, dtype=torch.uint8, pin_memory=True)
            g = torch.empty(m, dtype=torch.uint8, device=dev)
            for name, src, dst in (("h2d_pinned", h, g), ("d2h_pinned", g, h)):
                dst.copy_(src, non_blocking=True)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(5):
                    dst.copy_(src, non_blocking=True)
                torch.cuda.synchronize()
                out[name + tag + "_GBs"] = round(5 * m / (time.perf_counter() - t0) / 1e9, 1)
        return out

    roofline["measured_peaks"] = measured_peaks()

    # ---- host link: checkpoint traffic of the timed strategy.  With the DMA tier the copies run on a side stream
    # beside the compute stream; the rate below is what the step needs from the link (bytes moved over the step's
    # wall time), next to what one state-sized pinned copy achieves on this machine.
    link_bytes = int(st.d2h_bytes + st.h2d_bytes)
    host_link = {"tier": "none" if not link_bytes else ("direct (kernels write and read the mapped pinned block)" if host_direct else "dma (hipMemcpyAsync on the copy stream)"),
                 "bytes_per_step": link_bytes, "transfers_per_step": int(st.n_d2h + st.n_h2d), "message_bytes": Ms,
                 "sustained_GBs_over_the_step": round(link_bytes / sec / 1e9, 3),
                 "pinned_copy_of_one_state_GBs": {"h2d": roofline["measured_peaks"]["h2d_pinned_one_state_GBs"],
                                                  "d2h": roofline["measured_peaks"]["d2h_pinned_one_state_GBs"]},
                 "link_time_if_serial_ms": round(link_bytes / max(1e-9, roofline["measured_peaks"]["d2h_pinned_one_state_GBs"]) / 1e6, 3)}

    # ---- "max trainable T" and the 10x-sequence-length comparison ------------------------------------
    # Budget = what Standard BPTT needs for a tenth of this workload's T.  Under that same budget: the largest T each
    # strategy can train (closed form from snn_bytes_required, square-root intervals), and Double Checkpointing
    # actually run at the full T -- ten times Standard's length -- with intervals chosen for that budget, its time
    # per time step next to Standard's.
    long_seq = None
    if not args.no_long:
        progress("10x-sequence-length comparison")
        T_std = max(1, w.T // 10)
        cfg_std = snn.make_config(w.n_in, list(w.n_hidden), w.n_out, T_std, w.B)
        ref_budget = snn.snn_bytes_required(cfg_std, snn.SNN_STANDARD, T_std)

        def fits(sid, T, Cc, Ff, bud):
            cfgT = snn.make_config(w.n_in, list(w.n_hidden), w.n_out, T, w.B)
            need = snn.snn_bytes_required(cfgT, sid, T, Cc, Ff)
            return 0 < need <= bud

        def t_max(sid, bud):
            lo, hi = 0, 1
            while fits(sid, hi, 0, 0, bud) and hi < (1 << 26):
                lo, hi = hi, hi * 2
            while hi - lo > 1:
                mid = (lo + hi) // 2
                if fits(sid, mid, 0, 0, bud):
                    lo = mid
                else:
                    hi = mid
            return lo
        names = (("standard", snn.SNN_STANDARD), ("chunk", snn.SNN_CHUNK), ("remote", snn.SNN_REMOTE), ("double", snn.SNN_DOUBLE))
        tmax = {name: t_max(sid, ref_budget) for name, sid in names}
        tmax_cfg = {name: t_max(sid, budget) for name, sid in names} if budget else None

        def need_at(sid, T):
            return snn.snn_bytes_required(snn.make_config(w.n_in, list(w.n_hidden), w.n_out, T, w.B), sid, T, 0, 0)
        Ts = [w.T * m for m in (1, 2, 4, 8, 16, 32)]
        bytes_vs_T = {"T": Ts}
        for name, sid in names + (("hier", snn.SNN_HIER),):
            bytes_vs_T[name] = [int(need_at(sid, T)) for T in Ts]
        long_seq = {"budget_bytes": ref_budget, "budget_is": f"what Standard BPTT needs at T={T_std}", "t_max_under_budget": tmax,
                    "t_max_under_the_configuration_budget": tmax_cfg, "hbm_activation_bytes_vs_T": bytes_vs_T}
        try:
            CL, FL = snn.snn_suggest_intervals(net.cfg, snn.SNN_DOUBLE, w.T, ref_budget)
        except snn.SnnError:
            CL = FL = 0
        if CL:
            need_long = snn.snn_bytes_required(net.cfg, snn.SNN_DOUBLE, w.T, CL, FL)
            long_seq.update({"double_T": w.T, "double_coarse": CL, "double_fine": FL, "double_bytes_required": need_long})

            def step_long():
                net.snn_bind_inputs(x, y, w.T)
                return net.snn_bptt(snn.SNN_DOUBLE, CL, FL, ref_budget, want_stats=False)
            step_long()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.long_reps):
                step_long()
            torch.cuda.synchronize()
            sec_long = (time.perf_counter() - t0) / args.long_reps
            xs_, n_std = x[:T_std].contiguous() if hasattr(x, "contiguous") else np.ascontiguousarray(x[:T_std]), 3

            def step_std():
                net.snn_bind_inputs(xs_, y, T_std)
                net.snn_bptt(snn.SNN_STANDARD, 0, 0, ref_budget, want_stats=False)
            for _ in range(2):
                step_std()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(n_std):
                step_std()
            torch.cuda.synchronize()
            sec_std = (time.perf_counter() - t0) / n_std
            long_seq.update({"double_ms_per_step": round(sec_long * 1e3, 3),
                             "double_us_per_timestep": round(sec_long / w.T * 1e6, 4),
                             "standard_T": T_std, "standard_ms_per_step": round(sec_std * 1e3, 3),
                             "standard_us_per_timestep": round(sec_std / T_std * 1e6, 4),
                             "time_per_timestep_ratio_double_over_standard": round((sec_long / w.T) / (sec_std / T_std), 4),
                             "sequence_length_ratio": round(w.T / T_std, 2)})

    cpu = None
    if not args.no_cpu_baseline:
        progress("CPU baseline (oracle)")
        import oracle
        # the box's share of host cores: OMP_NUM_THREADS is set to it on the GPU machine (os.cpu_count() shows the
        # whole machine); the oracle parallelises over batch elements
        host_cores = os.cpu_count() or 1
        cores = max(1, min(host_cores, int(os.environ.get("OMP_NUM_THREADS", "16")), w.B))

        def time_oracle(Tc, nthreads, max_reps, min_wall):
            xs = np.ascontiguousarray(d["in_spikes"][:Tc])
            wall, reps, used = 0.0, 0, nthreads
            while reps < max_reps and (reps < 1 or wall < min_wall):
                t0 = time.perf_counter()
                r = oracle.bptt(w.n_in, list(w.n_hidden), w.n_out, d["W_in"], d["W_rec"], d["W_out"], xs, d["labels"],
                                alpha=w.alpha, beta=w.beta, theta=w.theta, surr_beta=w.surr_beta, rec_mask=d.get("rec_mask"),
                                dtype=np.float32, nthreads=nthreads)
                wall += time.perf_counter() - t0
                reps += 1
                used = r.stats.get("threads_used", nthreads) or nthreads
            return reps * w.B * Tc * w.neurons / wall, wall, reps, used
        # bounded samples: a prefix of the sequence sized from the network (about 10-30 s of CPU work in all)
        per_step = w.B * sum(n * (pn + 2 * n) for pn, n in zip([w.n_in] + list(w.n_hidden[:-1]), w.n_hidden))  # ~MACs per step
        T_all = int(max(2, min(w.T, 4e10 / per_step)))
        T_one = int(max(2, min(w.T, 4e9 / per_step)))
        v_all, wall_all, reps_all, used = time_oracle(T_all, cores, 6, 1.5)
        v_one, wall_one, reps_one, _ = time_oracle(T_one, 1, 3, 1.5)
        cpu = {"value": round(v_all, 1), "unit": "neuron-timesteps/s", "cores": int(used), "kind": "oracle",
               "one_thread_value": round(v_one, 1), "host_cpu_count": host_cores,
               "sample": f"oracle fp32 Standard BPTT (fwd+bwd), full batch: first {T_all} of {w.T} steps with {used} threads "
                         f"({reps_all} repetitions, {wall_all:.2f} s wall), first {T_one} steps with 1 thread "
                         f"({reps_one} repetitions, {wall_one:.2f} s wall); time is linear in T"}

    out = {
        "metric": "BPTT neuron-timesteps/sec (fwd+bwd) at fixed HBM budget", "value": round(nts / sec, 1),
        "unit": "neuron-timesteps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec * 1e3, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic" if not args.host_inputs else "synthetic, inputs handed over from host memory every step",
        "config": {"workload": w.name, "T": w.T, "batch": w.B, "strategy": args.strategy, "coarse_interval": C,
                   "fine_interval": F, "hbm_budget_bytes": budget,
                   "hbm_activation_bytes": int(st.bytes_states + st.bytes_spikes + st.bytes_workspace),
                   "hbm_activation_bytes_min": int(snn.snn_bytes_required(net.cfg, SID[args.strategy], w.T, C, F)),
                   "hbm_state_bytes": int(st.bytes_states), "state_slots_hbm": slots,
                   "state_slots_hbm_allocated": int(st.local_state_slots), "state_slots_host": rslots,
                   "recurrent_density": w.rec_density, "surrogate_window": args.surr_window, "spike_tier": args.spike_tier,
                   "hbm_spike_bytes": int(st.bytes_spikes), "host_spike_bytes": int(st.bytes_host_spikes),
                   "spike_link_bytes_per_step": int(st.spike_d2h_bytes + st.spike_h2d_bytes),
                   "firing_rate": [round(r, 4) for r in rates], "input_rate": round(in_rate, 4),
                   "same_intervals_under_the_smallest_budget": tight,
                   "forward_pass_kept_currents_of_steps": max(0, w.T - int(st.refwd_current_steps)) if args.strategy == "double" else 0,
                   "steps_per_pass": {"forward": int(st.fwd_steps), "re_forward_1": int(st.refwd1_steps),
                                      "re_forward_2": int(st.refwd2_steps), "backward": int(st.bwd_steps),
                                      "recompute_steps_whose_currents_were_computed": int(st.refwd_current_steps)},
                   "other_strategies_neuron_timesteps_per_s": others},
        "roofline": roofline, "cpu_baseline": cpu, "host_link": host_link, "long_sequence": long_seq,
    }
    print(json.dumps(out))
    net.snn_destroy()


if __name__ == "__main__":
    main()
