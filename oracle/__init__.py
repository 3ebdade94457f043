"""CPU oracle for LIF-SNN BPTT under the paper's checkpointing strategies.

TEST INFRASTRUCTURE ONLY.  This package wraps ``snn_oracle.c`` (plain C, built
twice: fp32 and fp64) with ctypes.  It is independent of the GPU library: it
imports nothing from it and shares no code with it.  Only the tests, the smoke
check and the benchmark's CPU-baseline leg may use it.

The model, the backward equations and the four storage schedules (Fig. 1 of
the paper; Sections "Standard Checkpointing", "Remote Checkpointing", "Double
Checkpointing") are documented at the top of ``snn_oracle.c``.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "snn_oracle.c")

STANDARD, CHUNK, REMOTE, DOUBLE, HIER = 0, 1, 2, 3, 4
HEAVISIDE, SMOOTH = 0, 1

EVENT_NAMES = {1: "SAVE_LOCAL", 2: "SAVE_REMOTE", 3: "LOAD_REMOTE", 4: "REFWD1",
               5: "KEEP_FINE", 6: "REFWD2", 7: "BACKWARD", 8: "SAVE_BATCH", 9: "LOAD_BATCH"}


def _lib_path(suffix: str) -> str:
    return os.path.join(_HERE, f"libsnn_oracle_{suffix}.so")


def build(force: bool = False) -> None:
    """Compile the oracle with gcc (fp32 and fp64 variants).  No fused multiply-add."""
    for real, suffix in (("float", "f32"), ("double", "f64")):
        out = _lib_path(suffix)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
            continue
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC", "-shared",
               f"-DREAL={real}", f"-DSUFFIX={suffix}", "-o", out, _SRC, "-lm"]
        subprocess.run(cmd, check=True)


class _Cfg(C.Structure):
    _fields_ = [("n_in", C.c_int32), ("n_layers", C.c_int32), ("n_out", C.c_int32),
                ("T", C.c_int32), ("B", C.c_int32), ("n_hidden", C.POINTER(C.c_int32)),
                ("alpha", C.c_double), ("beta", C.c_double), ("theta", C.c_double),
                ("surr_beta", C.c_double), ("mode", C.c_int32), ("forced", C.c_int32),
                ("strategy", C.c_int32), ("C", C.c_int32), ("F", C.c_int32),
                ("nthreads", C.c_int32), ("forced_states", C.c_int32), ("surr_window", C.c_double)]


class _Stats(C.Structure):
    _fields_ = [("fwd_steps", C.c_int64), ("refwd1_steps", C.c_int64), ("refwd2_steps", C.c_int64),
                ("bwd_steps", C.c_int64), ("remote_writes", C.c_int64), ("remote_reads", C.c_int64),
                ("local_slots", C.c_int64), ("remote_slots", C.c_int64), ("n_events", C.c_int64),
                ("threads_used", C.c_int32)]


_libs: dict = {}


def _lib(dtype) -> tuple:
    suffix = "f32" if np.dtype(dtype) == np.float32 else "f64"
    if suffix not in _libs:
        build()
        lib = C.CDLL(_lib_path(suffix))
        fn = getattr(lib, f"oracle_bptt_{suffix}")
        fn.restype = C.c_int
        _libs[suffix] = fn
    return _libs[suffix]


@dataclass
class Result:
    loss: float
    ubar: np.ndarray                       # [B, n_out]
    spikes: list                           # per hidden layer [T, B, N_l] (0/1, or real in smooth mode)
    v: list | None                         # per hidden layer [T, B, N_l] or None
    dW_in: list | None = None
    dW_rec: list | None = None
    dW_out: np.ndarray | None = None
    stats: dict = field(default_factory=dict)
    events: list = field(default_factory=list)   # [(name, a, b)] schedule of batch element 0


def _ptr_array(arrs, ctype):
    PT = C.POINTER(ctype)
    out = (PT * len(arrs))()
    for i, a in enumerate(arrs):
        out[i] = a.ctypes.data_as(PT) if a is not None else PT()
    return out


def bptt(n_in, n_hidden, n_out, W_in, W_rec, W_out, in_spikes, labels, *,
         alpha=0.9, beta=0.9, theta=1.0, surr_beta=10.0, dtype=np.float32,
         strategy=STANDARD, coarse=0, fine=0, mode=HEAVISIDE, forced_spikes=None,
         forced_v=None, rec_mask=None, backward=True, want_v=False, nthreads=1,
         want_events=False, surr_window=0.0) -> Result:
    """Run the oracle: forward, loss and (optionally) the backward pass.

    W_in[l]: [N_{l-1}, N_l], W_rec[l]: [N_l, N_l], W_out: [N_L, n_out] (row = presynaptic neuron);
    in_spikes: uint8 [T, B, n_in]; labels: int [B].  ``forced_spikes`` (list of [T, B, N_l]) makes
    the forward pass read the hidden spike trains instead of thresholding; ``forced_v`` (same
    shapes, needs ``forced_spikes``, full storage only) also fixes the membrane potentials, so that
    the backward pass can be evaluated in double precision on an fp32 forward trajectory.
    ``surr_window`` w > 0 cuts the surrogate derivative to zero wherever |v - theta| >= w.
    """
    dt = np.dtype(dtype)
    ct = C.c_float if dt == np.float32 else C.c_double
    L = len(n_hidden)
    in_spikes = np.ascontiguousarray(in_spikes, dtype=np.uint8)
    T, B, nin = in_spikes.shape
    assert nin == n_in
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    assert labels.shape == (B,) and labels.min() >= 0 and labels.max() < n_out
    pre = [n_in] + list(n_hidden[:-1])
    Wi = [np.ascontiguousarray(w, dtype=dt) for w in W_in]
    Wr = [np.ascontiguousarray(w, dtype=dt) for w in W_rec]
    Wo = np.ascontiguousarray(W_out, dtype=dt)
    for l in range(L):
        assert Wi[l].shape == (pre[l], n_hidden[l]) and Wr[l].shape == (n_hidden[l], n_hidden[l])
    assert Wo.shape == (n_hidden[-1], n_out)
    nh = np.asarray(n_hidden, dtype=np.int32)
    cfg = _Cfg(n_in, L, n_out, T, B, nh.ctypes.data_as(C.POINTER(C.c_int32)), alpha, beta, theta,
               surr_beta, mode, 1 if forced_spikes is not None else 0, strategy, coarse, fine, nthreads,
               1 if forced_v is not None else 0, surr_window)
    if forced_spikes is not None:
        spikes = [np.ascontiguousarray(s, dtype=dt).copy() for s in forced_spikes]
    else:
        spikes = [np.zeros((T, B, n), dtype=dt) for n in n_hidden]
    if forced_v is not None:
        assert forced_spikes is not None
        v = [np.ascontiguousarray(a, dtype=dt).copy() for a in forced_v]
    else:
        v = [np.zeros((T, B, n), dtype=dt) for n in n_hidden] if want_v else None
    ubar = np.zeros((B, n_out), dtype=dt)
    loss = C.c_double(0.0)
    dWi = [np.zeros_like(w) for w in Wi] if backward else [None] * L
    dWr = [np.zeros_like(w) for w in Wr] if backward else [None] * L
    dWo = np.zeros_like(Wo) if backward else None
    masks = None
    if rec_mask is not None:
        masks = [None if m is None else np.ascontiguousarray(m, dtype=np.uint8) for m in rec_mask]
    stats = _Stats()
    evcap = 0
    evbuf = None
    if want_events:
        evcap = 8 * (T + 8)
        evbuf = np.zeros((evcap, 3), dtype=np.int32)
    rc = _lib(dt)(
        C.byref(cfg), _ptr_array(Wi, ct), _ptr_array(Wr, ct), Wo.ctypes.data_as(C.POINTER(ct)),
        _ptr_array(masks, C.c_uint8) if masks is not None else None,
        in_spikes.ctypes.data_as(C.POINTER(C.c_uint8)), labels.ctypes.data_as(C.POINTER(C.c_int32)),
        _ptr_array(spikes, ct), _ptr_array(v, ct) if v is not None else None,
        ubar.ctypes.data_as(C.POINTER(ct)), C.byref(loss), 1 if backward else 0,
        _ptr_array(dWi, ct), _ptr_array(dWr, ct),
        dWo.ctypes.data_as(C.POINTER(ct)) if dWo is not None else None,
        C.byref(stats), evbuf.ctypes.data_as(C.POINTER(C.c_int32)) if evbuf is not None else None,
        C.c_int64(evcap))
    if rc != 0:
        raise ValueError("oracle_bptt: invalid arguments")
    events = []
    if want_events:
        assert stats.n_events <= evcap
        events = [(EVENT_NAMES[int(c)], int(a), int(b)) for c, a, b in evbuf[: stats.n_events]]
    st = {k: int(getattr(stats, k)) for k, _ in _Stats._fields_}
    return Result(float(loss.value), ubar, spikes, v, dWi if backward else None,
                  dWr if backward else None, dWo, st, events)
