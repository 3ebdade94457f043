"""Seeded synthetic inputs for the LIF-SNN BPTT workloads.

This module only draws random numbers and shapes them: weights, recurrent
masks, Bernoulli input spike trains and labels.  It holds none of the method's
arithmetic and is the only code shared by the CPU oracle's tests and the GPU
library's tests/benchmark, so that both sides see identical arrays.

The paper evaluates on spiking datasets that it only cites (Results section);
these i.i.d. Bernoulli spike trains of the same shape (e.g. 700 input channels,
20 classes) stand in for them.

Draw order for one seed (numpy ``default_rng(seed)``): W_in^1, W_rec^1, ...,
W_in^L, W_rec^L, W_out, recurrent masks (layer order), inputs, labels.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    n_in: int
    n_hidden: tuple
    n_out: int
    T: int
    B: int
    p_in: float                 # Bernoulli rate of the input spikes
    p_hidden: float = 0.05      # rate assumed for hidden layers in the weight scale
    gain: float = 1.0           # multiplies every weight's standard deviation
    rec_density: float = 1.0    # fraction of recurrent synapses that exist
    seed: int = 0
    alpha: float = 0.9
    beta: float = 0.9
    theta: float = 1.0
    surr_beta: float = 10.0

    @property
    def neurons(self) -> int:
        return int(sum(self.n_hidden))

    def neuron_timesteps(self) -> int:
        return self.B * self.T * self.neurons


# The five benchmark configurations (index = position in the configs list).
# ``gain`` for configs 2 and 4 is the value that tunes the hidden firing rate
# to about 5 %; it was found with the oracle (see oracle/calibrate_gain.py).
CONFIGS = {
    0: Workload("cfg0_tiny_32-64-10", 32, (64,), 10, T=50, B=2, p_in=0.05, seed=0),
    1: Workload("cfg1_classifier_700-256-256-20", 700, (256, 256), 20, T=1000, B=32, p_in=0.02, seed=1),
    2: Workload("cfg2_wide_700-3x1024-20", 700, (1024, 1024, 1024), 20, T=10000, B=64, p_in=0.01,
                gain=0.156, seed=2),
    3: Workload("cfg3_long_128-2x512-10", 128, (512, 512), 10, T=100000, B=16, p_in=0.01, seed=3),
    4: Workload("cfg4_large_1024-4x8192-100", 1024, (8192,) * 4, 100, T=5000, B=32, p_in=0.02,
                gain=0.2175, rec_density=0.1, seed=4),
}


def config(idx: int, **overrides) -> Workload:
    return replace(CONFIGS[idx], **overrides)


def generate(w: Workload, dtype=np.float32) -> dict:
    """Draw every array of one workload.  Returns a dict with W_in, W_rec (lists),
    W_out, rec_mask (list or None), in_spikes uint8 [T,B,n_in], labels int32 [B]."""
    rng = np.random.default_rng(w.seed)
    pre = [w.n_in] + list(w.n_hidden[:-1])
    W_in, W_rec = [], []
    for l, n in enumerate(w.n_hidden):
        p_pre = w.p_in if l == 0 else w.p_hidden
        std_in = w.gain * 2.0 / np.sqrt(pre[l] * p_pre)
        std_rec = w.gain * 2.0 / np.sqrt(n * w.p_hidden)
        W_in.append((rng.standard_normal((pre[l], n)) * std_in).astype(dtype))
        W_rec.append((rng.standard_normal((n, n)) * std_rec).astype(dtype))
    std_out = w.gain * 2.0 / np.sqrt(w.n_hidden[-1] * w.p_hidden)
    W_out = (rng.standard_normal((w.n_hidden[-1], w.n_out)) * std_out).astype(dtype)
    rec_mask = None
    if w.rec_density < 1.0:
        rec_mask = []
        for l, n in enumerate(w.n_hidden):
            m = (rng.random((n, n)) < w.rec_density).astype(np.uint8)
            rec_mask.append(m)
            W_rec[l] = W_rec[l] * m.astype(dtype)
    # drawn in blocks of time steps (same stream as one big draw, bounded temporary memory)
    in_spikes = np.empty((w.T, w.B, w.n_in), dtype=np.uint8)
    blk = max(1, (1 << 24) // max(1, w.B * w.n_in))
    for t0 in range(0, w.T, blk):
        t1 = min(w.T, t0 + blk)
        in_spikes[t0:t1] = rng.random((t1 - t0, w.B, w.n_in)) < w.p_in
    labels = rng.integers(0, w.n_out, size=w.B).astype(np.int32)
    return dict(W_in=W_in, W_rec=W_rec, W_out=W_out, rec_mask=rec_mask,
                in_spikes=in_spikes, labels=labels)


def forced_spike_trains(w: Workload, rates, seed: int | None = None) -> list:
    """I.i.d. Bernoulli hidden spike trains at exact per-layer rates (uint8 [T,B,N_l]);
    used by kernel micro-benchmarks that need a controlled activity level."""
    rng = np.random.default_rng(w.seed + 1000 if seed is None else seed)
    return [(rng.random((w.T, w.B, n)) < r).astype(np.uint8) for n, r in zip(w.n_hidden, rates)]
