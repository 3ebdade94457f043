"""Finds the scalar weight gain that tunes the hidden firing rate of a workload to a target
(configurations 2 and 4 ask for about 5 %).  Uses only the oracle's forward pass on a short prefix;
the result is recorded in synth.CONFIGS.  Usage: python -m oracle.calibrate_gain <config> [rate] [T] [B]"""
import sys

import numpy as np

import oracle
import synth


def measured_rates(w):
    d = synth.generate(w)
    r = oracle.bptt(w.n_in, list(w.n_hidden), w.n_out, d["W_in"], d["W_rec"], d["W_out"], d["in_spikes"], d["labels"],
                    alpha=w.alpha, beta=w.beta, theta=w.theta, dtype=np.float32, backward=False, nthreads=8)
    return [float(s.mean()) for s in r.spikes]


def calibrate(idx, target=0.05, T=200, B=4, hidden=None):
    lo, hi = 0.01, 1.0
    over = dict(T=T, B=B)
    if hidden:
        over["n_hidden"] = hidden
    for _ in range(14):
        mid = (lo * hi) ** 0.5
        rates = measured_rates(synth.config(idx, gain=mid, **over))
        mean = float(np.mean(rates))
        print(f"gain {mid:.4f} -> rates {[round(r, 4) for r in rates]}")
        if mean > target:
            hi = mid
        else:
            lo = mid
    return (lo * hi) ** 0.5


if __name__ == "__main__":
    idx = int(sys.argv[1])
    target = float(sys.argv[2]) if len(sys.argv) > 2 else 0.05
    T = int(sys.argv[3]) if len(sys.argv) > 3 else 200
    B = int(sys.argv[4]) if len(sys.argv) > 4 else 4
    print("gain =", round(calibrate(idx, target, T, B), 4))
