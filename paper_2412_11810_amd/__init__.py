"""Thin ctypes binding over libsnn_mi355x.so (the C ABI declared in include/snn.h).

Argument marshalling only: every step of the hot path runs in the HIP kernels of
the library.  There is no CPU fallback: if the library is missing or no GPU is
present, the calls raise.  Function names mirror the C entry points.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsnn_mi355x.so")

SNN_STANDARD, SNN_CHUNK, SNN_REMOTE, SNN_DOUBLE, SNN_HIER = 0, 1, 2, 3, 4
SNN_W_IN, SNN_W_REC, SNN_W_OUT = 0, 1, 2
SNN_OK, SNN_E_INVAL, SNN_E_BUDGET, SNN_E_HIP, SNN_E_HOSTMEM, SNN_E_STATE = range(6)
SNN_MAX_LAYERS = 4
STATUS_NAMES = ["SNN_OK", "SNN_E_INVAL", "SNN_E_BUDGET", "SNN_E_HIP", "SNN_E_HOSTMEM", "SNN_E_STATE"]
OP_NAMES = {1: "SAVE_LOCAL", 2: "SAVE_REMOTE", 3: "LOAD_REMOTE", 4: "REFWD1", 5: "KEEP_FINE",
            6: "REFWD2", 7: "BACKWARD", 8: "SAVE_BATCH", 9: "LOAD_BATCH"}

EXPORTS = ["snn_init", "snn_set_weights", "snn_forward", "snn_bptt", "snn_bind_inputs", "snn_grads",
           "snn_get_spikes", "snn_get_readout", "snn_debug_states", "snn_bytes_required",
           "snn_state_slots", "snn_schedule", "snn_last_error", "snn_destroy", "snn_debug_copy",
           "snn_suggest_intervals", "snn_debug_currents", "snn_get_state", "snn_forward_noalloc"]


class snn_config(C.Structure):
    _fields_ = [("n_in", C.c_int32), ("n_layers", C.c_int32), ("n_hidden", C.c_int32 * SNN_MAX_LAYERS),
                ("n_out", C.c_int32), ("T", C.c_int32), ("batch", C.c_int32), ("alpha", C.c_float),
                ("beta_out", C.c_float), ("theta", C.c_float), ("surr_beta", C.c_float),
                ("surr_window", C.c_float), ("device", C.c_int32), ("spike_tier", C.c_int32), ("stream", C.c_void_p)]


class snn_stats(C.Structure):
    _fields_ = [("ms_total", C.c_float), ("ms_forward", C.c_float), ("ms_backward_total", C.c_float),
                ("ms_recompute", C.c_float), ("ms_adjoint", C.c_float), ("ms_dw", C.c_float),
                ("ms_fwd_seq", C.c_float), ("ms_fwd_currents", C.c_float), ("ms_up_gemm", C.c_float),
                ("ms_bwd_stage", C.c_float), ("ms_fwd_stage", C.c_float), ("ms_scan", C.c_float),
                ("bytes_states", C.c_int64), ("bytes_spikes", C.c_int64), ("bytes_workspace", C.c_int64),
                ("bytes_host", C.c_int64), ("d2h_bytes", C.c_int64), ("h2d_bytes", C.c_int64),
                ("n_d2h", C.c_int32), ("n_h2d", C.c_int32), ("spike_d2h_bytes", C.c_int64),
                ("spike_h2d_bytes", C.c_int64), ("bytes_host_spikes", C.c_int64), ("fwd_steps", C.c_int64),
                ("refwd1_steps", C.c_int64), ("refwd2_steps", C.c_int64), ("bwd_steps", C.c_int64),
                ("refwd_current_steps", C.c_int64),
                ("local_state_slots", C.c_int32), ("remote_state_slots", C.c_int32),
                ("firing_rate", C.c_float * SNN_MAX_LAYERS)]

    def as_dict(self) -> dict:
        d = {k: getattr(self, k) for k, _ in self._fields_ if k != "firing_rate"}
        d["firing_rate"] = list(self.firing_rate)
        return d


class SnnError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{STATUS_NAMES[status] if 0 <= status < 6 else status}: {text}")
        self.status = status


_lib = None


def lib() -> C.CDLL:
    """Load the shared library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} not built: run `python -m paper_2412_11810_amd.build`")
        # One HIP runtime per process: PyTorch ships its own libamdhip64 (same SONAME as the system
        # one).  Loading it first makes this library bind to that copy, so torch tensors, streams
        # and this library share one runtime; a second runtime could not open the GPU.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
        L.snn_init.argtypes = [C.POINTER(snn_config), C.POINTER(vp)]
        L.snn_set_weights.argtypes = [vp, C.c_int, C.c_int, vp, vp]
        L.snn_forward.argtypes = [vp, vp, vp, i32, C.POINTER(C.c_float)]
        L.snn_forward_noalloc.argtypes = [vp, vp, vp, i32, C.POINTER(C.c_float)]
        L.snn_bptt.argtypes = [vp, C.c_int, i32, i32, sz, C.POINTER(snn_stats)]
        L.snn_bind_inputs.argtypes = [vp, vp, vp, i32]
        L.snn_grads.argtypes = [vp, C.c_int, C.c_int, vp, sz]
        L.snn_get_spikes.argtypes = [vp, C.c_int, vp]
        L.snn_get_readout.argtypes = [vp, vp, vp]
        L.snn_debug_states.argtypes = [vp, vp]
        L.snn_get_state.argtypes = [vp, C.c_int, i32, vp]
        L.snn_debug_copy.argtypes = [vp, vp, vp, sz]
        L.snn_debug_currents.argtypes = [vp, C.POINTER(vp), i32, i32, C.POINTER(C.c_float)]
        L.snn_bytes_required.argtypes = [C.POINTER(snn_config), C.c_int, i32, i32, i32]
        L.snn_bytes_required.restype = sz
        L.snn_suggest_intervals.argtypes = [C.POINTER(snn_config), C.c_int, i32, sz, C.POINTER(i32), C.POINTER(i32)]
        L.snn_state_slots.argtypes = [C.c_int, i32, i32, i32, C.POINTER(i32)]
        L.snn_state_slots.restype = i32
        L.snn_schedule.argtypes = [C.c_int, i32, i32, i32, vp, i64]
        L.snn_schedule.restype = i64
        L.snn_last_error.argtypes = [vp]
        L.snn_last_error.restype = C.c_char_p
        L.snn_destroy.argtypes = [vp]
        L.snn_destroy.restype = None
        for name in ("snn_init", "snn_set_weights", "snn_forward", "snn_bptt", "snn_bind_inputs", "snn_grads",
                     "snn_get_spikes", "snn_get_readout", "snn_debug_states", "snn_debug_copy", "snn_debug_currents",
                     "snn_get_state", "snn_forward_noalloc"):
            getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def make_config(n_in, n_hidden, n_out, T, batch, alpha=0.9, beta_out=0.9, theta=1.0, surr_beta=10.0,
                device=0, stream=None, surr_window=0.0, spike_tier=0) -> snn_config:
    cfg = snn_config()
    cfg.n_in, cfg.n_layers, cfg.n_out, cfg.T, cfg.batch = n_in, len(n_hidden), n_out, T, batch
    for i, n in enumerate(n_hidden):
        cfg.n_hidden[i] = n
    cfg.alpha, cfg.beta_out, cfg.theta, cfg.surr_beta = alpha, beta_out, theta, surr_beta
    cfg.surr_window = surr_window
    cfg.device = device
    cfg.spike_tier = spike_tier
    cfg.stream = stream
    return cfg


def snn_bytes_required(cfg: snn_config, strategy: int, T: int, coarse: int = 0, fine: int = 0) -> int:
    return int(lib().snn_bytes_required(C.byref(cfg), strategy, T, coarse, fine))


def snn_suggest_intervals(cfg: snn_config, strategy: int, T: int, hbm_budget_bytes: int = 0):
    c, f = C.c_int32(0), C.c_int32(0)
    st = lib().snn_suggest_intervals(C.byref(cfg), strategy, T, hbm_budget_bytes, C.byref(c), C.byref(f))
    if st != SNN_OK:
        raise SnnError(st, "no plan of this strategy fits the budget" if st == SNN_E_BUDGET else "invalid arguments")
    return int(c.value), int(f.value)


def snn_state_slots(strategy: int, T: int, coarse: int = 0, fine: int = 0):
    r = C.c_int32(0)
    n = lib().snn_state_slots(strategy, T, coarse, fine, C.byref(r))
    return int(n), int(r.value)


def snn_schedule(strategy: int, T: int, coarse: int = 0, fine: int = 0) -> list:
    n = lib().snn_schedule(strategy, T, coarse, fine, None, 0)
    if n < 0:
        raise SnnError(SNN_E_INVAL, "invalid strategy/intervals")
    buf = np.zeros((n, 3), dtype=np.int32)
    lib().snn_schedule(strategy, T, coarse, fine, buf.ctypes.data, n)
    return [(OP_NAMES[int(o)], int(a), int(b)) for o, a, b in buf]


def _ptr(x):
    """Address of a numpy array (host) or a torch tensor (host or device)."""
    if x is None:
        return None
    if isinstance(x, np.ndarray):
        assert x.flags["C_CONTIGUOUS"]
        return x.ctypes.data
    assert x.is_contiguous()
    return x.data_ptr()


class Snn:
    """One library context.  Methods are the C entry points with the context bound."""

    def __init__(self, cfg: snn_config):
        self._h = C.c_void_p()
        self.cfg = cfg
        self._keep = []
        st = lib().snn_init(C.byref(cfg), C.byref(self._h))
        if st != SNN_OK:
            text = lib().snn_last_error(self._h).decode() if self._h else "snn_init failed"
            if self._h:
                lib().snn_destroy(self._h)
                self._h = C.c_void_p()
            raise SnnError(st, text)

    def _check(self, st: int):
        if st != SNN_OK:
            raise SnnError(st, lib().snn_last_error(self._h).decode())

    def snn_set_weights(self, kind: int, layer: int, w, mask=None):
        if isinstance(w, np.ndarray):
            w = np.ascontiguousarray(w, dtype=np.float32)
        if isinstance(mask, np.ndarray):
            mask = np.ascontiguousarray(mask, dtype=np.uint8)
        self._check(lib().snn_set_weights(self._h, kind, layer, _ptr(w), _ptr(mask)))

    @staticmethod
    def _check_inputs(in_spikes, labels):
        """The C ABI takes raw pointers: the element types must already be right (uint8 spikes, int32 labels)."""
        for name, a, want in (("in_spikes", in_spikes, "uint8"), ("labels", labels, "int32")):
            if str(a.dtype).replace("torch.", "") != want:
                raise TypeError(f"{name} must be {want}, got {a.dtype}")

    def snn_bind_inputs(self, in_spikes, labels, T: int):
        self._check_inputs(in_spikes, labels)
        self._check(lib().snn_bind_inputs(self._h, _ptr(in_spikes), _ptr(labels), T))

    def snn_forward(self, in_spikes, labels, T: int) -> float:
        loss = C.c_float(0)
        self._check_inputs(in_spikes, labels)
        self._check(lib().snn_forward(self._h, _ptr(in_spikes), _ptr(labels), T, C.byref(loss)))
        return float(loss.value)

    def snn_forward_noalloc(self, in_spikes, labels, T: int) -> float:
        loss = C.c_float(0)
        self._check_inputs(in_spikes, labels)
        self._check(lib().snn_forward_noalloc(self._h, _ptr(in_spikes), _ptr(labels), T, C.byref(loss)))
        return float(loss.value)

    def snn_bptt(self, strategy: int, coarse: int = 0, fine: int = 0, hbm_budget_bytes: int = 0,
                 want_stats: bool = True):
        st = snn_stats()
        self._check(lib().snn_bptt(self._h, strategy, coarse, fine, hbm_budget_bytes,
                                   C.byref(st) if want_stats else None))
        return st if want_stats else None

    def _shape(self, kind: int, layer: int):
        nh = [self.cfg.n_hidden[i] for i in range(self.cfg.n_layers)]
        if kind == SNN_W_OUT:
            return (nh[-1], self.cfg.n_out)
        if kind == SNN_W_IN:
            return ((self.cfg.n_in if layer == 0 else nh[layer - 1]), nh[layer])
        return (nh[layer], nh[layer])

    def snn_grads(self, kind: int, layer: int = 0) -> np.ndarray:
        out = np.empty(self._shape(kind, layer), dtype=np.float32)
        self._check(lib().snn_grads(self._h, kind, layer, out.ctypes.data, out.size))
        return out

    def snn_get_spikes(self, layer: int, T: int) -> np.ndarray:
        out = np.empty((T, self.cfg.batch, self.cfg.n_hidden[layer]), dtype=np.uint8)
        self._check(lib().snn_get_spikes(self._h, layer, out.ctypes.data))
        return out

    def snn_get_readout(self):
        ubar = np.empty((self.cfg.batch, self.cfg.n_out), dtype=np.float32)
        loss = C.c_float(0)
        self._check(lib().snn_get_readout(self._h, ubar.ctypes.data, C.addressof(loss)))
        return ubar, float(loss.value)

    def snn_get_state(self, layer: int, t: int) -> np.ndarray:
        out = np.empty((self.cfg.batch, self.cfg.n_hidden[layer]), dtype=np.float32)
        self._check(lib().snn_get_state(self._h, layer, t, out.ctypes.data))
        return out

    def snn_debug_states(self, T: int) -> np.ndarray:
        sn = sum(self.cfg.n_hidden[i] for i in range(self.cfg.n_layers))
        out = np.empty((T, self.cfg.batch, sn), dtype=np.float32)
        self._check(lib().snn_debug_states(self._h, out.ctypes.data))
        return out

    def snn_debug_copy(self, src, dst, nbytes: int):
        self._check(lib().snn_debug_copy(self._h, _ptr(src), _ptr(dst), nbytes))

    def snn_debug_currents(self, hidden, chunk: int, reps: int = 1) -> float:
        """hidden: one array / tensor [T][B][N_l] of 0/1 bytes per hidden layer (None: keep the layer's spikes).
        Returns the mean time in ms of one pass of the current kernels over the bound sequence."""
        L = self.cfg.n_layers
        arr = (C.c_void_p * L)()
        keep = []
        for l in range(L):
            h = hidden[l] if l < len(hidden) else None
            if h is None:
                arr[l] = None
                continue
            if isinstance(h, np.ndarray):
                h = np.ascontiguousarray(h, dtype=np.uint8)
            keep.append(h)
            arr[l] = _ptr(h)
        ms = C.c_float(0.0)
        self._check(lib().snn_debug_currents(self._h, arr, chunk, reps, C.byref(ms)))
        return float(ms.value)

    def snn_destroy(self):
        if self._h:
            lib().snn_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.snn_destroy()
        except Exception:
            pass


def from_workload(w, data: dict, T: int | None = None, device: int = 0, stream=None,
                  surr_window: float = 0.0, spike_tier: int = 0) -> Snn:
    """Context for a synth.Workload with its weights loaded."""
    cfg = make_config(w.n_in, list(w.n_hidden), w.n_out, T or w.T, w.B, w.alpha, w.beta, w.theta,
                      w.surr_beta, device, stream, surr_window, spike_tier)
    net = Snn(cfg)
    for l in range(len(w.n_hidden)):
        net.snn_set_weights(SNN_W_IN, l, data["W_in"][l])
        net.snn_set_weights(SNN_W_REC, l, data["W_rec"][l],
                            None if data.get("rec_mask") is None else data["rec_mask"][l])
    net.snn_set_weights(SNN_W_OUT, 0, data["W_out"])
    return net
