"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element.

Bar: spike trains bit-exact (mismatches tolerated only at steps where the oracle's |v - theta| < 1e-5;
they are counted and printed -- with the shared summation order the expected count is 0); fp32
gradients within 1e-4 of max|grad| per tensor; all GPU strategies bit-identical to each other."""
import numpy as np
import pytest

import oracle
import synth

pytestmark = pytest.mark.gpu

snn = pytest.importorskip("paper_2412_11810_amd")

GRAD_TOL = 1e-4


def _oracle(w, d, **kw):
    return oracle.bptt(w.n_in, list(w.n_hidden), w.n_out, d["W_in"], d["W_rec"], d["W_out"], d["in_spikes"],
                       d["labels"], alpha=w.alpha, beta=w.beta, theta=w.theta, surr_beta=w.surr_beta,
                       rec_mask=d.get("rec_mask"), dtype=np.float32, **kw)


def _oracle_f64_on_f32_trajectory(w, d, ref32, nthreads, window=0.0):
    """Gradient reference: the oracle's backward pass in double precision, evaluated on the fp32 forward
    trajectory (spike trains and membrane potentials of the fp32 oracle, which the GPU reproduces bit for
    bit).  The fp32 oracle itself cannot serve at 1e-4: its sequential fp32 gradient sums over tens of
    thousands of terms are off by ~2e-4 (it disagrees with itself by that much between thread counts)."""
    return oracle.bptt(w.n_in, list(w.n_hidden), w.n_out, d["W_in"], d["W_rec"], d["W_out"], d["in_spikes"],
                       d["labels"], alpha=w.alpha, beta=w.beta, theta=w.theta, surr_beta=w.surr_beta,
                       rec_mask=d.get("rec_mask"), dtype=np.float64,
                       forced_spikes=[s.astype(np.float64) for s in ref32.spikes],
                       forced_v=[v.astype(np.float64) for v in ref32.v], nthreads=nthreads, surr_window=window)


def _gpu_grads(net, L):
    return ([net.snn_grads(snn.SNN_W_IN, l) for l in range(L)], [net.snn_grads(snn.SNN_W_REC, l) for l in range(L)],
            net.snn_grads(snn.SNN_W_OUT, 0))


def _check_spikes(net, w, ref, tag):
    bad_total = 0
    for l in range(len(w.n_hidden)):
        got = net.snn_get_spikes(l, w.T)
        exp = ref.spikes[l].astype(np.uint8)
        mism = got != exp
        if mism.any():
            near = np.abs(ref.v[l] - w.theta) < 1e-5
            first_t = int(np.argwhere(mism)[0][0])
            # only the first divergent step can be judged: later ones follow from it
            assert np.all(near[first_t][mism[first_t]]), f"{tag}: layer {l} spikes differ away from the threshold at t={first_t + 1}"
            bad_total += int(mism.sum())
    near_steps = sum(int((np.abs(ref.v[l] - w.theta) < 1e-5).any(axis=(1, 2)).sum()) for l in range(len(w.n_hidden)))
    print(f"[{tag}] steps with |v-theta|<1e-5 in the oracle: {near_steps}; spike mismatches: {bad_total}")
    return bad_total


def _check_grads(gpu, ref, tag):
    gi, gr, go = gpu
    worst = 0.0
    for name, a, b in ([(f"dW_in[{l}]", gi[l], ref.dW_in[l]) for l in range(len(gi))] +
                       [(f"dW_rec[{l}]", gr[l], ref.dW_rec[l]) for l in range(len(gr))] + [("dW_out", go, ref.dW_out)]):
        scale = np.abs(b).max()
        if scale == 0:  # e.g. no recurrent contribution when T = 1
            assert not np.any(a), f"{tag}: {name} must be exactly zero"
            continue
        err = np.abs(a - b).max() / scale
        worst = max(worst, err)
        assert err <= GRAD_TOL, f"{tag}: {name} max rel err {err:.3e}"
    print(f"[{tag}] worst gradient error / max|grad| = {worst:.3e}")


def _identical(a, b):
    return all(np.array_equal(x, y) for x, y in zip(a[0] + a[1] + [a[2]], b[0] + b[1] + [b[2]]))


def _full_parity(w, strategies, nthreads=8, check_states=True, window=0.0, probe_states=()):
    d = synth.generate(w)
    # the fp32 oracle supplies the forward trajectory (its own gradients are not the reference: see
    # test_gradient_reference_for_the_gpu_parity_bar among the oracle pins)
    ref = _oracle(w, d, want_v=True, nthreads=nthreads, surr_window=window, backward=False)
    ref64 = _oracle_f64_on_f32_trajectory(w, d, ref, nthreads, window)
    net = snn.from_workload(w, d, surr_window=window)
    try:
        loss = net.snn_forward(d["in_spikes"], d["labels"], w.T)
        assert _check_spikes(net, w, ref, w.name + " forward") == 0
        assert abs(loss - ref.loss) <= 2e-5 * max(1.0, abs(ref.loss))
        ubar, _ = net.snn_get_readout()
        assert np.allclose(ubar, ref.ubar, rtol=1e-5, atol=1e-5)
        if check_states:
            v = net.snn_debug_states(w.T)
            off = 0
            for l, n in enumerate(w.n_hidden):
                assert np.array_equal(v[:, :, off:off + n], ref.v[l]), f"membrane potentials of layer {l} differ"
                off += n
        first = None
        for strat, C, F in strategies:
            tag = f"{w.name} strat={strat} C={C} F={F}"
            st = net.snn_bptt(strat, C, F)
            assert _check_spikes(net, w, ref, tag) == 0
            g = _gpu_grads(net, len(w.n_hidden))
            _check_grads(g, ref64, tag)
            for (pl, pt) in probe_states:  # rebuilt from the stored spike trains, whatever the strategy stored
                assert np.array_equal(net.snn_get_state(pl, pt), ref.v[pl][pt - 1]), f"{tag}: v of layer {pl} at t={pt}"
            if first is None:
                first = g
            else:
                assert _identical(g, first), f"{tag}: gradients not bit-identical to the first strategy"
            assert st.fwd_steps == w.T and st.bwd_steps == w.T
            rates = [float(ref.spikes[l].mean()) for l in range(len(w.n_hidden))]
            assert np.allclose(list(st.firing_rate)[:len(rates)], rates, atol=1e-6)
        return first, ref
    finally:
        net.snn_destroy()


def test_hand_trace_on_gpu():
    """The 3-neuron, 5-step hand trace, through the GPU library."""
    W_in = np.array([[1.5, 0.5, 0], [0, 0.75, 0.25]], np.float32)
    W_rec = np.array([[0, 0.5, 1.0], [-0.5, 0, 0.5], [0.25, -1.0, 0]], np.float32)
    W_out = np.array([[1, 0], [0, 1], [0.5, 0.5]], np.float32)
    x = np.array([[1, 0], [0, 1], [1, 1], [0, 0], [1, 0]], np.uint8)[:, None, :].copy()
    y = np.array([0], np.int32)
    net = snn.Snn(snn.make_config(2, [3], 2, 5, 1, alpha=0.5, beta_out=0.5))
    net.snn_set_weights(snn.SNN_W_IN, 0, W_in)
    net.snn_set_weights(snn.SNN_W_REC, 0, W_rec)
    net.snn_set_weights(snn.SNN_W_OUT, 0, W_out)
    loss = net.snn_forward(x, y, 5)
    v = net.snn_debug_states(5)[:, 0, :]
    assert np.array_equal(v, np.array([[1.5, 0.5, 0], [-0.25, 1.5, 1.25], [1.125, 0, 0.375], [-0.4375, 0.5, 1.1875],
                                       [1.53125, -0.25, -0.40625]], np.float32))
    assert np.array_equal(net.snn_get_spikes(0, 5)[:, 0, :], [[1, 0, 0], [0, 1, 1], [1, 0, 0], [0, 0, 1], [1, 0, 0]])
    assert abs(loss - 0.450937) < 2e-6
    net.snn_bptt(snn.SNN_DOUBLE, 3, 2)
    assert np.allclose(net.snn_grads(snn.SNN_W_OUT), [[-0.340284, 0.340284], [-0.136113, 0.136113], [-0.245004, 0.245004]], atol=2e-6)
    net.snn_destroy()


def test_config0_all_strategies():
    _full_parity(synth.config(0), [(snn.SNN_STANDARD, 0, 0), (snn.SNN_CHUNK, 0, 10), (snn.SNN_CHUNK, 0, 7),
                                   (snn.SNN_REMOTE, 10, 0), (snn.SNN_REMOTE, 13, 0), (snn.SNN_DOUBLE, 20, 5),
                                   (snn.SNN_DOUBLE, 17, 4), (snn.SNN_DOUBLE, 50, 1), (snn.SNN_CHUNK, 0, 50),
                                   (snn.SNN_DOUBLE, 0, 0), (snn.SNN_CHUNK, 0, 0), (snn.SNN_HIER, 2, 5),
                                   (snn.SNN_HIER, 1, 7), (snn.SNN_HIER, 3, 10), (snn.SNN_HIER, 0, 0)], nthreads=1)


def test_ragged_three_layer_net():
    """Layer widths that are not multiples of the wavefront, several words per layer, a ragged tail."""
    w = synth.Workload("ragged_70-100-72-130-7", 70, (100, 72, 130), 7, T=61, B=3, p_in=0.1, gain=0.5, seed=11)
    _full_parity(w, [(snn.SNN_STANDARD, 0, 0), (snn.SNN_CHUNK, 0, 9), (snn.SNN_REMOTE, 8, 0), (snn.SNN_DOUBLE, 16, 5),
                     (snn.SNN_HIER, 2, 4), (snn.SNN_HIER, 1, 3)], nthreads=3)


def test_masked_recurrent_weights():
    w = synth.Workload("masked_40-96-96-5", 40, (96, 96), 5, T=40, B=4, p_in=0.1, gain=0.8, rec_density=0.2, seed=12)
    _full_parity(w, [(snn.SNN_STANDARD, 0, 0), (snn.SNN_DOUBLE, 12, 4)], nthreads=4)


def test_wide_layer_two_neurons_per_thread():
    """1024-wide layers (the width of configuration 2) at a short T: more than one neuron per thread."""
    w = synth.config(2, T=24, B=3)
    _full_parity(w, [(snn.SNN_STANDARD, 0, 0), (snn.SNN_DOUBLE, 10, 4)], nthreads=3)


def test_surrogate_window():
    """Surrogate derivative with compact support (zero where |v - theta| >= w): every adjoint kernel
    (register-stationary, cross-workgroup for 512 and 1024 neurons, streaming for wider layers) against
    the oracle with the same window, and the window must actually cut: the gradients differ from the
    unwindowed ones while dW_out (which passes through no threshold) stays the same bit for bit."""
    w0 = synth.config(0)
    strategies = [(snn.SNN_STANDARD, 0, 0), (snn.SNN_CHUNK, 0, 7), (snn.SNN_REMOTE, 13, 0), (snn.SNN_DOUBLE, 17, 4),
                  (snn.SNN_HIER, 2, 5)]
    g_win, ref = _full_parity(w0, strategies, nthreads=1, window=0.5)
    g_all, _ = _full_parity(w0, strategies[:1], nthreads=1)
    inside = np.mean([float((np.abs(v - w0.theta) < 0.5).mean()) for v in ref.v])
    print(f"[window 0.5] fraction of (t, b, neuron) inside the window: {inside:.3f}")
    assert 0.0 < inside < 1.0
    assert np.array_equal(g_win[2], g_all[2])
    assert not np.array_equal(g_win[1][0], g_all[1][0])
    wide = synth.Workload("window_40-300-1100-5", 40, (300, 1100), 5, T=20, B=3, p_in=0.1, gain=0.6, seed=21)
    _full_parity(wide, [(snn.SNN_STANDARD, 0, 0), (snn.SNN_DOUBLE, 8, 3)], nthreads=3, window=0.4)
    _full_parity(synth.config(2, T=24, B=3), [(snn.SNN_STANDARD, 0, 0), (snn.SNN_CHUNK, 0, 5)], nthreads=3, window=0.4)


def test_chip_wide_adjoint_valu_version(monkeypatch):
    """Layers of 257..1024 neurons run the chip-wide adjoint recurrence on the matrix cores by default; the VALU
    version of the same kernel (SNN_WS_KERNEL=valu) must meet the same bar against the oracle."""
    monkeypatch.setenv("SNN_WS_KERNEL", "valu")
    w = synth.Workload("wsvalu_24-512-300-6", 24, (512, 300), 6, T=18, B=5, p_in=0.1, gain=0.6, seed=23)
    _full_parity(w, [(snn.SNN_STANDARD, 0, 0), (snn.SNN_DOUBLE, 8, 3)], nthreads=5, check_states=False)
    _full_parity(synth.config(2, T=12, B=3), [(snn.SNN_STANDARD, 0, 0), (snn.SNN_CHUNK, 0, 5)], nthreads=3, check_states=False)
    monkeypatch.delenv("SNN_WS_KERNEL")


@pytest.mark.parametrize("hidden,B,T,C,F,density", [((300, 520), 5, 43, 8, 3, 1.0), ((1024,), 20, 30, 10, 4, 1.0),
                                                     ((2048, 2048), 3, 26, 8, 4, 0.1)])
def test_forward_pass_keeps_currents_for_double(hidden, B, T, C, F, density, monkeypatch):
    """Double with the currents cache: the forward pass of layers above 256 neurons leaves the synaptic currents of
    the last coarse segments in the cache -- the last segment without a budget, as many whole segments as fit under a
    budget, every step under a generous one -- and Re-Forward_1 of those segments computes none (counted in the
    statistics).  Ragged last segment, three sequential kernels (one workgroup per batch element, sliced, sliced over
    compressed rows).  Against the oracle, and bit-identical to the step that keeps nothing (SNN_KEEP_CURRENTS=0)."""
    w = synth.Workload("keep_" + "x".join(map(str, hidden)), 40, hidden, 6, T=T, B=B, p_in=0.1, gain=0.6,
                       rec_density=density, seed=61 + B)
    if density < 1.0:
        monkeypatch.setenv("SNN_CSR", "1")
    if len(hidden) == 1:  # checkpoints through the copy engine (states this small go out by direct stores otherwise)
        monkeypatch.setenv("SNN_HOST_TIER", "dma")
    first, _ = _full_parity(w, [(snn.SNN_STANDARD, 0, 0), (snn.SNN_DOUBLE, C, F)], nthreads=8, check_states=False)
    d = synth.generate(w)
    cfg = snn.make_config(w.n_in, list(w.n_hidden), w.n_out, w.T, w.B)
    last = T - ((T - 1) // C) * C                      # steps of the (ragged) last coarse segment
    tight = snn.snn_bytes_required(cfg, snn.SNN_DOUBLE, T, C, F)  # (one chunk buffer, no cache: both come first)
    slot = 4 * B * sum(hidden)
    seen = {}
    for tag, keep, budget in (("none", "0", 0), ("last", "1", 0), ("one_more", "1", tight + (last + C + len(hidden) * F) * slot + slot // 2),
                              ("all", "1", tight + 2 * T * slot)):
        monkeypatch.setenv("SNN_KEEP_CURRENTS", keep)
        net = snn.from_workload(w, d)
        try:
            net.snn_bind_inputs(d["in_spikes"], d["labels"], w.T)
            st = net.snn_bptt(snn.SNN_DOUBLE, C, F, budget)
            assert _identical(first, _gpu_grads(net, len(hidden))), tag
            seen[tag] = int(st.refwd_current_steps)
            if budget:
                assert st.bytes_states + st.bytes_spikes + st.bytes_workspace <= budget
        finally:
            net.snn_destroy()
    monkeypatch.delenv("SNN_KEEP_CURRENTS")
    assert seen["none"] == T and seen["last"] == T - last and seen["all"] == 0, seen
    assert seen["one_more"] == T - last - C, seen


def test_forward_stage_of_wide_masked_layers_in_one_launch(monkeypatch):
    """Wide layers over compressed rows with the dense current kernel: the feed-forward currents for the next pipeline
    stage ride in the launch of a stage's sequential parts (k_fwd_stage_csr).  Two tiles (64 + 9 steps), two layers:
    against the oracle (spikes, potentials, gradients), and bit-identical to the separate launches (SNN_FWD_FUSE=0)."""
    w = synth.Workload("fwdstage_2048x2048", 40, (2048, 2048), 6, T=73, B=3, p_in=0.1, gain=0.6, rec_density=0.1, seed=77)
    monkeypatch.setenv("SNN_CSR", "1")
    monkeypatch.setenv("SNN_CURRENTS", "dense")
    first, _ = _full_parity(w, [(snn.SNN_STANDARD, 0, 0), (snn.SNN_DOUBLE, 16, 4)], nthreads=8)
    monkeypatch.setenv("SNN_FWD_FUSE", "0")
    d = synth.generate(w)
    net = snn.from_workload(w, d)
    try:
        net.snn_bind_inputs(d["in_spikes"], d["labels"], w.T)
        net.snn_bptt(snn.SNN_STANDARD, 0, 0)
        assert _identical(first, _gpu_grads(net, 2))
        spikes_sep = [net.snn_get_spikes(l, w.T) for l in range(2)]
    finally:
        net.snn_destroy()
    monkeypatch.delenv("SNN_FWD_FUSE")
    net = snn.from_workload(w, d)
    try:
        net.snn_forward(d["in_spikes"], d["labels"], w.T)
        for l in range(2):
            assert np.array_equal(net.snn_get_spikes(l, w.T), spikes_sep[l])
    finally:
        net.snn_destroy()


def test_weight_gradient_kernel_follows_the_rates():
    """Networks with layers wider than 256 start with the dense contraction of the weight gradients and move to the
    tiled event-driven kernel when the previous step's presynaptic activity was below 8 % (configuration 2's widths
    at its 5 %), and back above it: consecutive training steps on the same inputs must give the same bits, at a low
    and at a high rate, and both match the oracle."""
    for gain, lo, hi in ((0.156, 0.0, 0.08), (0.3, 0.08, 1.0)):
        w = synth.config(2, T=16, B=8)
        w = synth.Workload(w.name, w.n_in, w.n_hidden, w.n_out, T=16, B=8, p_in=w.p_in, gain=gain, seed=w.seed)
        first, ref = _full_parity(w, [(snn.SNN_STANDARD, 0, 0), (snn.SNN_CHUNK, 0, 5), (snn.SNN_DOUBLE, 8, 3)], nthreads=8,
                                  check_states=False)
        rate = float(np.mean([s.mean() for s in ref.spikes]))
        assert lo <= rate < hi, f"gain {gain}: hidden rate {rate:.3f} is outside the regime this case is meant for"


@pytest.mark.parametrize("hidden,B,T", [((520, 300), 20, 12), ((1024,), 32, 10), ((640, 640, 640), 64, 9)])
def test_chip_wide_adjoint_two_batch_groups_per_workgroup(hidden, B, T, monkeypatch):
    """Layers of 257..1024 neurons with an even number of 16-element batch groups: a workgroup of the chip-wide
    adjoint recurrence can serve two groups half a step apart with the same registers of W_rec (the library does so
    only when asked, SNN_WS_KERNEL=pair), or own 64 rows with eight wavefronts (where the stage's layers would not
    fit one launch otherwise, or SNN_WS_KERNEL=rows64).  A ragged second group, widths below the padded reduction
    length, a ragged last row block, three layers in one launch: against the oracle, and bit-identical to the kernel
    with 32 rows and one group per workgroup (SNN_WS_KERNEL=single)."""
    w = synth.Workload("ws2_" + "x".join(map(str, hidden)), 40, hidden, 6, T=T, B=B, p_in=0.1, gain=0.6, seed=41 + B)
    monkeypatch.setenv("SNN_WS_KERNEL", "pair")
    first, _ = _full_parity(w, [(snn.SNN_STANDARD, 0, 0), (snn.SNN_DOUBLE, 6, 3)], nthreads=8, check_states=False)
    d = synth.generate(w)
    flat = lambda g: list(g[0]) + list(g[1]) + [g[2]]
    for mode in ("single", "rows64"):  # one group and 32 rows per workgroup; 64 rows (eight wavefronts)
        monkeypatch.setenv("SNN_WS_KERNEL", mode)
        net = snn.from_workload(w, d)
        try:
            net.snn_bind_inputs(d["in_spikes"], d["labels"], w.T)
            net.snn_bptt(snn.SNN_STANDARD, 0, 0)
            other = _gpu_grads(net, len(hidden))
        finally:
            net.snn_destroy()
        for a, b in zip(flat(first), flat(other)):
            assert np.array_equal(a, b), mode
    monkeypatch.delenv("SNN_WS_KERNEL")


@pytest.mark.parametrize("hidden,B,T", [((1088,), 5, 14), ((1152, 1088), 20, 10), ((1088,), 40, 8), ((4096,), 3, 9)])
def test_streamed_chip_wide_adjoint(hidden, B, T, monkeypatch):
    """Layers wider than 1024 neurons: the recurrence of the adjoint streams W_rec once per step for the whole
    batch (matrix cores, workgroups of 16 or 32 rows, batch in 1, 2 or 4 blocks of 16, a reduction range that is
    not a multiple of the prefetch ring).  Against the oracle, bit-identical between strategies, and within the
    tolerance of the one-workgroup-per-batch-element kernel it replaces."""
    w = synth.Workload("wide_" + "x".join(map(str, hidden)), 40, hidden, 7, T=T, B=B, p_in=0.1, seed=31 + B)
    first, _ = _full_parity(w, [(snn.SNN_STANDARD, 0, 0), (snn.SNN_CHUNK, 0, 4), (snn.SNN_DOUBLE, 8, 3)], nthreads=4)
    monkeypatch.setenv("SNN_WS_KERNEL", "stream")
    d = synth.generate(w)
    net = snn.from_workload(w, d)
    try:
        net.snn_bind_inputs(d["in_spikes"], d["labels"], w.T)
        net.snn_bptt(snn.SNN_STANDARD, 0, 0)
        other = _gpu_grads(net, len(hidden))
    finally:
        net.snn_destroy()
    monkeypatch.delenv("SNN_WS_KERNEL")
    flat = lambda g: list(g[0]) + list(g[1]) + [g[2]]
    for a, b in zip(flat(first), flat(other)):
        scale = float(np.max(np.abs(b))) or 1.0
        assert float(np.max(np.abs(a - b))) <= 1e-4 * scale


@pytest.mark.parametrize("hidden,B,T,force", [((2048, 2048), 3, 80, "0"), ((3072,), 3, 70, "0"), ((4096, 4096), 2, 20, "0"),
                                              ((512, 512), 5, 150, "8"), ((384,), 4, 100, "2")])
def test_sliced_sequential_forward_is_bitwise_neutral(hidden, B, T, force, monkeypatch):
    """Layers of 2048 neurons and more (narrower ones when SNN_SEQ_SLICES asks for it: 64-thread and 192-thread
    workgroups): the sequential part of the forward pass spreads the neurons
    of a batch element over several workgroups that exchange their spike words every step.  Spike trains, membrane
    potentials and gradients must be the very bits of the one-workgroup-per-batch-element kernel, and match the
    oracle."""
    w = synth.Workload("sliced_" + "x".join(map(str, hidden)), 50, hidden, 6, T=T, B=B, p_in=0.1, gain=0.7, seed=41 + B)
    d = synth.generate(w)
    L = len(hidden)
    got = {}
    for slices in ("auto", "1"):
        monkeypatch.setenv("SNN_SEQ_SLICES", "1" if slices == "1" else force)
        net = snn.from_workload(w, d)
        try:
            net.snn_bind_inputs(d["in_spikes"], d["labels"], w.T)
            states = net.snn_debug_states(w.T)
            net.snn_bptt(snn.SNN_CHUNK, 0, 16)
            got[slices] = (_gpu_grads(net, L), [net.snn_get_spikes(l, w.T) for l in range(L)], states)
        finally:
            net.snn_destroy()
    monkeypatch.delenv("SNN_SEQ_SLICES")
    assert _identical(got["auto"][0], got["1"][0])
    for a, b in zip(got["auto"][1], got["1"][1]):
        assert np.array_equal(a, b)
        assert a.sum() > 0
    assert np.array_equal(got["auto"][2].view(np.uint32), got["1"][2].view(np.uint32))
    _full_parity(w, [(snn.SNN_STANDARD, 0, 0), (snn.SNN_DOUBLE, 16, 5)], nthreads=4)


def test_current_kernels_on_forced_spike_trains(monkeypatch):
    """snn_debug_currents (the micro-benchmark entry): hidden spike trains at an exact rate replace the stored ones
    and every current kernel runs over them; a training step afterwards is unaffected (the forward pass rewrites
    the spike trains)."""
    w = synth.Workload("forced_60-300-280-5", 60, (300, 280), 5, T=40, B=6, p_in=0.1, gain=0.6, seed=23)
    d = synth.generate(w)
    hid = synth.forced_spike_trains(w, [0.1, 0.1])
    net = snn.from_workload(w, d)
    try:
        with pytest.raises(snn.SnnError):
            net.snn_debug_currents(hid, 8)  # nothing bound yet
        net.snn_bind_inputs(d["in_spikes"], d["labels"], w.T)
        for mode in ("gather", "mfma", "dense"):
            monkeypatch.setenv("SNN_CURRENTS", mode)
            assert net.snn_debug_currents(hid, 8, reps=2) > 0.0
        monkeypatch.delenv("SNN_CURRENTS")
        assert net.snn_debug_currents([None, hid[1]], 100) > 0.0
        with pytest.raises(snn.SnnError):
            net.snn_debug_currents(hid, 0)
    finally:
        net.snn_destroy()
    _full_parity(w, [(snn.SNN_STANDARD, 0, 0), (snn.SNN_CHUNK, 0, 7)], nthreads=2)


def test_wide_input_layer_with_stage_kernels():
    """3000 input channels in front of two 256-wide layers: the spike words and lists of the matrix-core current
    kernel still fit beside the sequential part of a forward stage, but no longer with eight wavefronts beside the
    adjoint recurrences, so the recompute work of later chunks moves to the launch between the stages."""
    w = synth.Workload("wide_in_3000-256-224-9", 3000, (256, 224), 9, T=70, B=4, p_in=0.03, gain=0.5, seed=27)
    _full_parity(w, [(snn.SNN_STANDARD, 0, 0), (snn.SNN_CHUNK, 0, 8), (snn.SNN_REMOTE, 16, 0), (snn.SNN_DOUBLE, 24, 5)],
                 nthreads=4)


def test_config1_full_size():
    """Configuration 1 at its full size (T = 1000, batch 32): Standard, Chunk(32), Remote(32) as the configuration
    lists, plus Double and Hier; single states through snn_get_state at a tile boundary, inside a tile and at T."""
    _full_parity(synth.config(1), [(snn.SNN_STANDARD, 0, 0), (snn.SNN_CHUNK, 0, 32), (snn.SNN_REMOTE, 32, 0),
                                   (snn.SNN_DOUBLE, 100, 10), (snn.SNN_HIER, 4, 32)], nthreads=8, check_states=True,
                 probe_states=[(0, 1), (1, 64), (0, 333), (1, 1000)])


def test_config2_widths_full_batch():
    """Configuration 2's widths at its full batch (64): the chip-wide adjoint recurrence with four batch groups and
    two layers' jobs per launch, full 64-row blocks in the current kernels, the wide weight-gradient tiles -- the
    launch shapes the benchmark times -- with gradients against the oracle."""
    w = synth.config(2, T=40)
    _full_parity(w, [(snn.SNN_STANDARD, 0, 0), (snn.SNN_DOUBLE, 20, 10), (snn.SNN_CHUNK, 0, 10)], nthreads=16,
                 check_states=True, probe_states=[(2, 40), (1, 17)])


def test_config4_widths_full_batch():
    """Configuration 4's widths at its full batch (32), masked recurrent matrices, with the library's own
    rate-driven choice of current kernel (nothing forced; the first step runs before any rate is known, the
    later ones after): gradients against the oracle."""
    w = synth.config(4, T=8)
    _full_parity(w, [(snn.SNN_DOUBLE, 4, 2), (snn.SNN_STANDARD, 0, 0), (snn.SNN_CHUNK, 0, 3)], nthreads=16,
                 check_states=True, probe_states=[(3, 8), (0, 5)])


def test_config4_widths_full_batch_high_activity():
    """The same network driven to 15-40 % hidden activity (weight gain 0.45), nothing forced: from the second training
    step on the rate-driven choice computes the recompute currents of the masked layers dense but still walks their
    compressed rows in the sequential forward part; gradients against the oracle, strategies bit-identical."""
    w = synth.config(4, T=8, gain=0.45)
    _full_parity(w, [(snn.SNN_DOUBLE, 4, 2), (snn.SNN_STANDARD, 0, 0), (snn.SNN_CHUNK, 0, 3)], nthreads=16,
                 check_states=True, probe_states=[(3, 8), (1, 3)])


def test_config3_width_reduced_length():
    w = synth.config(3, T=700, B=4)
    _full_parity(w, [(snn.SNN_CHUNK, 0, 27), (snn.SNN_DOUBLE, 316, 18)], nthreads=4, check_states=False)


def test_budget_and_argument_errors():
    w = synth.config(0)
    d = synth.generate(w)
    net = snn.from_workload(w, d)
    with pytest.raises(snn.SnnError) as e:
        net.snn_bptt(snn.SNN_STANDARD)
    assert e.value.status == snn.SNN_E_STATE
    net.snn_bind_inputs(d["in_spikes"], d["labels"], w.T)
    need = snn.snn_bytes_required(net.cfg, snn.SNN_STANDARD, w.T)
    with pytest.raises(snn.SnnError) as e:
        net.snn_bptt(snn.SNN_STANDARD, 0, 0, need - 1)
    assert e.value.status == snn.SNN_E_BUDGET
    st = net.snn_bptt(snn.SNN_STANDARD, 0, 0, need)
    assert st.bytes_states + st.bytes_spikes + st.bytes_workspace == need
    need_d = snn.snn_bytes_required(net.cfg, snn.SNN_DOUBLE, w.T, 10, 3)
    assert need_d < need
    st = net.snn_bptt(snn.SNN_DOUBLE, 10, 3, need_d)
    assert (st.n_d2h, st.n_h2d) == (4, 5) and st.remote_state_slots == 5
    assert st.refwd2_steps == w.T and st.refwd1_steps == 45
    with pytest.raises(snn.SnnError) as e:
        net.snn_bptt(snn.SNN_DOUBLE, 3, 5)
    assert e.value.status == snn.SNN_E_INVAL
    with pytest.raises(snn.SnnError):
        net.snn_bind_inputs(d["in_spikes"], d["labels"], w.T + 1)
    # labels are range-checked on the host before any kernel indexes the readout with them
    for bad in (w.n_out, -1):
        lab = d["labels"].copy()
        lab[1] = bad
        with pytest.raises(snn.SnnError) as e:
            net.snn_bind_inputs(d["in_spikes"], lab, w.T)
        assert e.value.status == snn.SNN_E_INVAL and "label" in str(e.value)
    with pytest.raises(TypeError):
        net.snn_bind_inputs(d["in_spikes"], d["labels"].astype(np.int64), w.T)
    net.snn_bind_inputs(d["in_spikes"], d["labels"], w.T)
    with pytest.raises(snn.SnnError) as e:
        net.snn_get_state(0, 1)  # no forward pass since the inputs were bound
    assert e.value.status == snn.SNN_E_STATE
    net.snn_bptt(snn.SNN_CHUNK, 0, 10)
    for bad_t in (0, w.T + 1):
        with pytest.raises(snn.SnnError) as e:
            net.snn_get_state(0, bad_t)
        assert e.value.status == snn.SNN_E_INVAL
    net.snn_destroy()


def test_graph_replay_follows_a_change_of_the_recurrent_mask():
    """A recorded training step holds the pointers it was recorded with, the recurrent mask among them.  Setting
    weights (with a mask, then without) between replays must give what an eager step gives, bit for bit: masked
    gradients are zero where the mask is, and a replay after the mask is dropped does not touch the freed mask."""
    w = synth.Workload("maskswap_40-96-96-5", 40, (96, 96), 5, T=40, B=4, p_in=0.1, gain=0.8, rec_density=0.3, seed=13)
    d = synth.generate(w)
    L = len(w.n_hidden)
    dense = [np.ascontiguousarray(d["W_rec"][l]) for l in range(L)]
    net = snn.Snn(snn.make_config(w.n_in, list(w.n_hidden), w.n_out, w.T, w.B))
    try:
        for l in range(L):
            net.snn_set_weights(snn.SNN_W_IN, l, d["W_in"][l])
            net.snn_set_weights(snn.SNN_W_REC, l, dense[l])          # no mask yet
        net.snn_set_weights(snn.SNN_W_OUT, 0, d["W_out"])
        net.snn_bind_inputs(d["in_spikes"], d["labels"], w.T)
        for phase in ("unmasked", "masked", "unmasked again"):
            if phase == "masked":
                for l in range(L):
                    net.snn_set_weights(snn.SNN_W_REC, l, dense[l], d["rec_mask"][l])
            elif phase == "unmasked again":
                for l in range(L):
                    net.snn_set_weights(snn.SNN_W_REC, l, dense[l])
            net.snn_bptt(snn.SNN_DOUBLE, 12, 4, want_stats=True)      # eager
            eager = _gpu_grads(net, L)
            for rep in range(2):
                net.snn_bptt(snn.SNN_DOUBLE, 12, 4, want_stats=False) # records, then replays
                assert _identical(_gpu_grads(net, L), eager), (phase, rep)
            for l in range(L):
                outside = eager[1][l][d["rec_mask"][l] == 0]
                assert (not outside.any()) == (phase == "masked"), phase
    finally:
        net.snn_destroy()


def test_suggested_intervals_train_within_the_budget():
    """Intervals picked by snn_suggest_intervals for a budget: the step runs inside that budget and gives the
    gradients of full storage bit for bit."""
    w = synth.config(1, T=1000, B=8)
    d = synth.generate(w)
    L = len(w.n_hidden)
    net = snn.from_workload(w, d)
    try:
        net.snn_bind_inputs(d["in_spikes"], d["labels"], w.T)
        net.snn_bptt(snn.SNN_STANDARD)
        ref = _gpu_grads(net, L)
        full = snn.snn_bytes_required(net.cfg, snn.SNN_STANDARD, w.T)
        for strat in (snn.SNN_CHUNK, snn.SNN_REMOTE, snn.SNN_DOUBLE, snn.SNN_HIER):
            for frac in (0.35, 0.6):
                budget = int(full * frac)
                C, F = snn.snn_suggest_intervals(net.cfg, strat, w.T, budget)
                st = net.snn_bptt(strat, C, F, budget)
                assert st.bytes_states + st.bytes_spikes + st.bytes_workspace <= budget
                assert _identical(_gpu_grads(net, L), ref), (strat, C, F)
    finally:
        net.snn_destroy()


def test_shorter_sequence_in_same_context_and_device_inputs():
    """A context sized for T serves shorter sequences; inputs may already live in device memory."""
    torch = pytest.importorskip("torch")
    w = synth.config(0)
    d = synth.generate(w)
    short = synth.config(0, T=23)
    ds = dict(d, in_spikes=np.ascontiguousarray(d["in_spikes"][:23]))
    ref = _oracle(short, ds, want_v=True)
    net = snn.from_workload(w, d)
    x = torch.from_numpy(ds["in_spikes"]).cuda()
    y = torch.from_numpy(ds["labels"]).cuda()
    net.snn_forward(x, y, 23)
    net.snn_bptt(snn.SNN_CHUNK, 0, 5)
    assert _check_spikes(net, short, ref, "short") == 0
    _check_grads(_gpu_grads(net, 1), _oracle_f64_on_f32_trajectory(short, ds, ref, 1), "short")
    net.snn_destroy()


def test_graph_replay_matches_eager():
    """snn_bptt without statistics replays a recorded HIP graph.  Every replay must give exactly what
    the eager (instrumented) call gives, also after other work ran in between and after the plan changed."""
    w = synth.config(1, T=200, B=8)
    d = synth.generate(w)
    net = snn.from_workload(w, d)
    net.snn_bind_inputs(d["in_spikes"], d["labels"], w.T)
    L = len(w.n_hidden)
    for strat, C, F in [(snn.SNN_DOUBLE, 50, 7), (snn.SNN_REMOTE, 32, 0), (snn.SNN_STANDARD, 0, 0)]:
        net.snn_bptt(strat, C, F, want_stats=True)              # eager
        ref = _gpu_grads(net, L)
        ref_spk = net.snn_get_spikes(1, w.T)
        for rep in range(3):
            net.snn_bptt(strat, C, F, want_stats=False)         # records on the first call, replays after
            assert _identical(_gpu_grads(net, L), ref), (strat, rep)
            assert np.array_equal(net.snn_get_spikes(1, w.T), ref_spk)
            net.snn_forward(d["in_spikes"], d["labels"], w.T)   # eager work between replays
            net.snn_bptt(snn.SNN_CHUNK, 0, 9, want_stats=True)  # a different plan, eager
    # new inputs through the same graph: the recording must not have baked any input in
    d2 = synth.generate(synth.config(1, T=200, B=8, seed=77))
    net.snn_bind_inputs(d2["in_spikes"], d2["labels"], w.T)
    net.snn_bptt(snn.SNN_STANDARD, 0, 0, want_stats=False)
    g_graph = _gpu_grads(net, L)
    net.snn_bptt(snn.SNN_STANDARD, 0, 0, want_stats=True)
    assert _identical(_gpu_grads(net, L), g_graph)
    net.snn_destroy()


def test_layer_pipelined_adjoint_is_bitwise_neutral(monkeypatch):
    """The adjoint pass runs its layers one chunk apart (layer l of chunk c together with layer l+1 of the
    chunk before it in time) when the budget has room for one chunk buffer per layer, and for layers of
    193..256 neurons the weight gradients of a stage ride in the next stage's launch (one more buffer) and so
    does the recompute of the next two chunks (two more buffers);
    otherwise, or with SNN_BWD_PIPE=0 / SNN_BWD_FUSE=0, it falls back step by step to finishing a chunk layer
    by layer.  Gradients must not differ by a bit, for every strategy, with chunks longer and shorter than the
    adjoint tile, three layers, and mixed kernel flavours."""
    cases = [(synth.config(1, T=300, B=6), [(snn.SNN_STANDARD, 0, 0), (snn.SNN_CHUNK, 0, 7), (snn.SNN_REMOTE, 32, 0),
                                             (snn.SNN_DOUBLE, 100, 10), (snn.SNN_HIER, 2, 16), (snn.SNN_CHUNK, 0, 290)]),
             (synth.Workload("pipe_50-200-256-230-7", 50, (200, 256, 230), 7, T=70, B=5, p_in=0.1, gain=0.5, seed=32),
              [(snn.SNN_STANDARD, 0, 0), (snn.SNN_CHUNK, 0, 9), (snn.SNN_DOUBLE, 30, 4), (snn.SNN_REMOTE, 1, 0)]),
             (synth.Workload("pipe_50-100-72-300-7", 50, (100, 72, 300), 7, T=45, B=3, p_in=0.1, gain=0.5, seed=31),
              [(snn.SNN_STANDARD, 0, 0), (snn.SNN_CHUNK, 0, 4), (snn.SNN_DOUBLE, 12, 5), (snn.SNN_REMOTE, 1, 0)])]
    modes = {"fused": {}, "fused_inter": {"SNN_PRE_IN_STAGE": "0"}, "pipelined": {"SNN_BWD_FUSE": "0"},
             "plain": {"SNN_BWD_PIPE": "0"}}
    for w, strategies in cases:
        d = synth.generate(w)
        L = len(w.n_hidden)
        fusable = all(192 < n <= 256 for n in w.n_hidden)
        got = {}
        for mode, env in modes.items():
            for k in ("SNN_BWD_FUSE", "SNN_BWD_PIPE", "SNN_PRE_IN_STAGE"):
                monkeypatch.delenv(k, raising=False)
            for k, v in env.items():
                monkeypatch.setenv(k, v)
            net = snn.from_workload(w, d)
            try:
                net.snn_bind_inputs(d["in_spikes"], d["labels"], w.T)
                for strat, C, F in strategies:
                    st = net.snn_bptt(strat, C, F)
                    got[(mode, strat, C, F)] = (_gpu_grads(net, L), st.local_state_slots, st.ms_bwd_stage)
                    if mode == "fused":
                        # budgets with room for fewer chunk buffers: same result, fewer slots
                        need = snn.snn_bytes_required(net.cfg, strat, w.T, C, F)
                        st2 = net.snn_bptt(strat, C, F, need)
                        assert _identical(_gpu_grads(net, L), got[(mode, strat, C, F)][0]), (w.name, strat, C, F)
                        assert st2.local_state_slots == snn.snn_state_slots(strat, w.T, C, F)[0]
                        chunk_len = {snn.SNN_CHUNK: F, snn.SNN_REMOTE: C, snn.SNN_DOUBLE: F, snn.SNN_HIER: F}.get(strat, 0)
                        st3 = net.snn_bptt(strat, C, F, need + (L - 1) * chunk_len * 4 * w.B * sum(w.n_hidden))
                        assert _identical(_gpu_grads(net, L), got[(mode, strat, C, F)][0]), (w.name, strat, C, F)
                        assert st3.ms_bwd_stage == 0 or strat == snn.SNN_STANDARD
                        # room for the fused weight-gradient update but not for recomputing ahead
                        st4 = net.snn_bptt(strat, C, F, need + L * chunk_len * 4 * w.B * sum(w.n_hidden))
                        assert _identical(_gpu_grads(net, L), got[(mode, strat, C, F)][0]), (w.name, strat, C, F)
                        assert (st4.ms_bwd_stage > 0) == fusable
                        net.snn_bptt(strat, C, F, want_stats=False)  # and through graph replay
                        assert _identical(_gpu_grads(net, L), got[(mode, strat, C, F)][0]), (w.name, strat, C, F)
            finally:
                net.snn_destroy()
        for strat, C, F in strategies:
            a, b, c, a2 = (got[(m, strat, C, F)] for m in ("fused", "pipelined", "plain", "fused_inter"))
            assert _identical(a[0], b[0]) and _identical(a[0], c[0]) and _identical(a[0], a2[0]), (w.name, strat, C, F)
            assert _identical(a[0], got[("fused",) + strategies[0]][0]), (w.name, strat, C, F)
            assert (a[2] > 0) == fusable and b[2] == 0 and c[2] == 0
            if strat != snn.SNN_STANDARD:
                # (Double with room to spare also keeps the currents of a coarse segment between its two recompute
                # passes, C more slots, except under the fused stage launches, which recompute ahead on their own)
                cache = lambda mode: C if (strat == snn.SNN_DOUBLE and C > F and not (fusable and mode.startswith("fused"))) else 0
                assert b[1] - cache("pipelined") > c[1] - cache("plain") == snn.snn_state_slots(strat, w.T, C, F)[0]
                assert (a[1] - cache("fused") > b[1] - cache("pipelined")) == fusable
    for k in ("SNN_BWD_FUSE", "SNN_BWD_PIPE", "SNN_PRE_IN_STAGE"):
        monkeypatch.delenv(k, raising=False)


def test_gather_and_matrix_core_currents_agree(monkeypatch):
    """The synaptic currents are computed either event by event (gather of the active rows), by the K = 1
    MFMA kernel that visits the rows active in a block of 16 (t, b) rows, or by its dense version that visits
    every presynaptic neuron for 64 (t, b) rows at a time (meant for matrices far beyond the L2; forced here).
    All add the same rows in the same order and must give the very same bits: spike trains, membrane
    potentials and gradients, for a dense-activity and a sparse-activity network and for layers that run
    outside the stage kernels (320 and 300 neurons: a ragged last block of columns, 70 inputs: a partial word)."""
    for w in (synth.config(1, T=150, B=6), synth.Workload("sparse_90-200-130-7", 90, (200, 130), 7, T=150, B=5, p_in=0.03, gain=0.3, seed=21),
              synth.Workload("mid_70-320-300-9", 70, (320, 300), 9, T=45, B=5, p_in=0.08, gain=0.6, seed=22)):
        d = synth.generate(w)
        L = len(w.n_hidden)
        got = {}
        for mode in ("gather", "mfma", "dense"):
            monkeypatch.setenv("SNN_CURRENTS", mode)
            net = snn.from_workload(w, d)
            try:
                net.snn_bind_inputs(d["in_spikes"], d["labels"], w.T)
                states = net.snn_debug_states(w.T)
                net.snn_bptt(snn.SNN_CHUNK, 0, 16)
                got[mode] = (_gpu_grads(net, L), [net.snn_get_spikes(l, w.T) for l in range(L)], states)
            finally:
                net.snn_destroy()
        for other in ("mfma", "dense"):
            assert _identical(got["gather"][0], got[other][0]), (w.name, other)
            for a, b in zip(got["gather"][1], got[other][1]):
                assert np.array_equal(a, b), (w.name, other)
            assert np.array_equal(got["gather"][2].view(np.uint32), got[other][2].view(np.uint32)), (w.name, other)
        assert sum(int(x.sum()) for x in got["gather"][1]) > 0, w.name
    monkeypatch.delenv("SNN_CURRENTS")


def test_event_driven_step_of_narrow_layers_is_bitwise_neutral(monkeypatch):
    """Layers of up to 256 neurons run the register-stationary chain (one FMA per presynaptic neuron whatever the
    activity); SNN_SEQ_KERNEL=gather sends them through the event-driven gather of the wide layers instead.  Both
    add the same weights in the same ascending order: spike trains, potentials and gradients must be identical,
    at a low and at a high firing rate."""
    for gain in (0.15, 1.0):
        w = synth.config(1, T=120, B=6, gain=gain)
        d = synth.generate(w)
        L = len(w.n_hidden)
        got = {}
        for mode in ("rs", "gather"):
            monkeypatch.setenv("SNN_SEQ_KERNEL", mode)
            net = snn.from_workload(w, d)
            try:
                net.snn_bind_inputs(d["in_spikes"], d["labels"], w.T)
                states = net.snn_debug_states(w.T)
                net.snn_bptt(snn.SNN_DOUBLE, 30, 6)
                got[mode] = (_gpu_grads(net, L), [net.snn_get_spikes(l, w.T) for l in range(L)], states)
            finally:
                net.snn_destroy()
        monkeypatch.delenv("SNN_SEQ_KERNEL")
        assert _identical(got["rs"][0], got["gather"][0]), gain
        for a, b in zip(got["rs"][1], got["gather"][1]):
            assert np.array_equal(a, b), gain
        assert np.array_equal(got["rs"][2].view(np.uint32), got["gather"][2].view(np.uint32)), gain
    _full_parity(w, [(snn.SNN_STANDARD, 0, 0), (snn.SNN_CHUNK, 0, 7)], nthreads=2)


@pytest.mark.parametrize("width,density", [(512, 1.0), (2048, 1.0), (1088, 1.0), (2048, 0.2)])
def test_barrier_timeout_is_reported_not_hung(monkeypatch, width, density):
    """The chip-wide adjoint kernels of wide layers (weights in registers up to 1024 neurons, streamed
    above, over compressed rows for a masked matrix) and the sliced sequential part of their forward pass (widths from 2048 that are multiples of 1024)
    synchronise their workgroups with a counting barrier
    that polls a bounded number of times.  With the limit forced to zero from the host every workgroup
    gives up at its first barrier: all kernels still run to completion, and snn_bptt reports the
    failure instead of returning gradients.  A context created afterwards works normally."""
    w = synth.Workload(f"wide_24-{width}-6", 24, (width,), 6, T=12, B=4, p_in=0.1, rec_density=density, seed=11)
    d = synth.generate(w)
    monkeypatch.setenv("SNN_WS_SPIN_LIMIT", "0")
    net = snn.from_workload(w, d)
    try:
        net.snn_bind_inputs(d["in_spikes"], d["labels"], w.T)
        with pytest.raises(RuntimeError, match="timed out"):
            net.snn_bptt(snn.SNN_STANDARD, 0, 0)
    finally:
        net.snn_destroy()
    monkeypatch.delenv("SNN_WS_SPIN_LIMIT")
    _full_parity(w, [(snn.SNN_STANDARD, 0, 0), (snn.SNN_CHUNK, 0, 5)], nthreads=1)


def test_host_tier_dma_and_direct_agree(monkeypatch):
    """Remote and Double keep their coarse checkpoints in pinned host memory.  Small states are written
    and read by the kernels themselves, larger ones travel by hipMemcpyAsync on the copy stream
    (SNN_HOST_TIER forces either way, read when the context is created).  Both ways must give the
    gradients of full storage bit for bit, eagerly and as a replayed graph."""
    w = synth.config(1, T=300, B=8)
    d = synth.generate(w)
    L = len(w.n_hidden)
    ref = None
    for tier in ("dma", "direct"):
        monkeypatch.setenv("SNN_HOST_TIER", tier)
        net = snn.from_workload(w, d)
        try:
            net.snn_bind_inputs(d["in_spikes"], d["labels"], w.T)
            if ref is None:
                net.snn_bptt(snn.SNN_STANDARD, 0, 0)
                ref = _gpu_grads(net, L)
            for strat, C, F in [(snn.SNN_REMOTE, 32, 0), (snn.SNN_DOUBLE, 70, 9), (snn.SNN_REMOTE, 300, 0)]:
                st = net.snn_bptt(strat, C, F)
                assert _identical(_gpu_grads(net, L), ref), (tier, strat, "eager")
                assert st.n_d2h == -(-w.T // C) - 1 and st.n_h2d == -(-w.T // C)
                for rep in range(2):
                    net.snn_bptt(strat, C, F, want_stats=False)
                    assert _identical(_gpu_grads(net, L), ref), (tier, strat, "graph", rep)
        finally:
            net.snn_destroy()


@pytest.mark.parametrize("T,B,strat,C,F", [(1, 1, 0, 0, 0), (1, 2, 3, 1, 1), (2, 1, 2, 1, 0), (65, 2, 1, 0, 64),
                                           (129, 1, 3, 64, 64), (130, 3, 2, 65, 0), (7, 5, 3, 7, 1),
                                           (130, 2, 4, 1, 3), (70, 1, 4, 2, 70), (33, 2, 4, 5, 2)])
def test_degenerate_sizes(T, B, strat, C, F):
    """One step, one batch element, intervals equal to T or to 1, tile and segment boundaries that
    do not line up (the forward tile is 64 steps)."""
    # a small gain keeps the readout away from softmax saturation (with one batch element and a
    # saturated softmax the fp32 loss gradient is pure rounding noise, whatever the implementation)
    w = synth.Workload("edge_20-48-33-4", 20, (48, 33), 4, T=T, B=B, p_in=0.15, gain=0.25, seed=5)
    _full_parity(w, [(snn.SNN_STANDARD, 0, 0), (strat, C, F)], nthreads=1)


@pytest.mark.parametrize("B", [12, 100, 128, 130])
def test_batch_sizes_of_the_weight_gradient_paths(B):
    """The weight-gradient contraction sums the products of one time step in fp32 (B/4 K-steps: a whole number
    of 4-K-step groups only when B is a multiple of 16) before the fp64 accumulation; more than 64 batch elements
    take the narrow tiles, more than 128 the event-by-event kernel.  All against the oracle, with the stage
    kernels (two layers of 193..256 neurons) and without (a narrower net)."""
    for hidden in ((200, 256), (90, 70)):
        w = synth.Workload(f"batch{B}_30-{hidden[0]}-{hidden[1]}-5", 30, hidden, 5, T=21, B=B, p_in=0.1, gain=0.5, seed=40 + B)
        _full_parity(w, [(snn.SNN_STANDARD, 0, 0), (snn.SNN_CHUNK, 0, 4), (snn.SNN_DOUBLE, 10, 3)], nthreads=8,
                     check_states=False)


def test_seeded_random_shapes():
    """Twenty seeded random networks (1-4 layers; widths that take the stage kernels, the narrow register-stationary
    kernels, the chip-wide and the streaming adjoint kernels, and mixtures), random T, batch, rates and intervals of
    every strategy: the same bar as everywhere else."""
    import random
    rng = random.Random(20241)
    for it in range(20):
        L = rng.choice([1, 2, 2, 3, 4])
        cls = rng.choice(["stage", "stage", "small", "mixed", "wide"])
        if cls == "stage":
            hidden = tuple(rng.randint(193, 256) for _ in range(L))
        elif cls == "small":
            hidden = tuple(rng.randint(3, 128) for _ in range(L))
        elif cls == "mixed":
            hidden = tuple(rng.choice([rng.randint(5, 256), rng.randint(257, 600)]) for _ in range(L))
        else:
            hidden = tuple(rng.randint(257, 1100) for _ in range(L))
        T, B = rng.randint(1, 150), rng.choice([1, 2, 3, 5, 8, 16, 17, 33])
        w = synth.Workload(f"random{it}", rng.randint(1, 130), hidden, rng.randint(1, 24), T=T, B=B,
                           p_in=rng.choice([0.02, 0.1, 0.3]), gain=rng.choice([0.3, 0.6, 1.0]), seed=2000 + it)
        strategies = [(snn.SNN_STANDARD, 0, 0)]
        for _ in range(3):
            s = rng.choice([snn.SNN_CHUNK, snn.SNN_REMOTE, snn.SNN_DOUBLE, snn.SNN_HIER])
            if s == snn.SNN_CHUNK:
                strategies.append((s, 0, rng.randint(1, T)))
            elif s == snn.SNN_REMOTE:
                strategies.append((s, rng.randint(1, T), 0))
            elif s == snn.SNN_DOUBLE:
                C = rng.randint(1, T)
                strategies.append((s, C, rng.randint(1, C)))
            else:
                strategies.append((s, rng.randint(1, 5), rng.randint(1, T)))
        print(f"[random {it}] hidden={hidden} n_in={w.n_in} n_out={w.n_out} T={T} B={B} {strategies}", flush=True)
        _full_parity(w, strategies, nthreads=min(8, B), check_states=(sum(hidden) * T * B < 4e6),
                     probe_states=[(L - 1, T), (0, max(1, T // 2))])


def _full_size_properties(idx, strategies, budget, prefix):
    """At a configuration's full size the oracle cannot run the whole step in test time.  Checked
    instead: (1) the forward pass is causal, so the first `prefix` steps of the full-length spike
    trains must equal, bit for bit, the oracle's spike trains for a sequence of that length; (2) every
    strategy gives bit-identical gradients; (3) the step respects the configuration's HBM budget."""
    w = synth.config(idx)
    d = synth.generate(w)
    short = synth.config(idx, T=prefix)
    ds = dict(d, in_spikes=np.ascontiguousarray(d["in_spikes"][:prefix]))
    ref = _oracle(short, ds, backward=False, nthreads=16)
    net = snn.from_workload(w, d)
    try:
        net.snn_bind_inputs(d["in_spikes"], d["labels"], w.T)
        first = None
        for strat, C, F, *own in strategies:
            # a fourth entry: this strategy's own budget ("min" = the smallest one its intervals can run in)
            bud = budget if not own else (snn.snn_bytes_required(net.cfg, strat, w.T, C, F) if own[0] == "min" else own[0])
            st = net.snn_bptt(strat, C, F, bud)
            assert st.bytes_states + st.bytes_spikes + st.bytes_workspace <= bud
            g = _gpu_grads(net, len(w.n_hidden))
            assert all(np.isfinite(x).all() for x in g[0] + g[1] + [g[2]])
            if first is None:
                first = g
                for l in range(len(w.n_hidden)):
                    got = net.snn_get_spikes(l, w.T)[:prefix]
                    assert np.array_equal(got, ref.spikes[l].astype(np.uint8)), f"layer {l}: prefix of the spike train differs"
                print(f"[{w.name}] rates {[round(float(r), 4) for r in list(st.firing_rate)[:len(w.n_hidden)]]}, "
                      f"step {st.ms_total:.1f} ms, activation bytes {st.bytes_states + st.bytes_spikes + st.bytes_workspace}")
            else:
                assert _identical(g, first), f"strategy {strat} ({C},{F}) differs from the first one at full size"
    finally:
        net.snn_destroy()


def test_config2_full_size_properties():
    """Configuration 2 (700 -> 3x1024 -> 20, T = 10 000, batch 64) under its 8 GB budget: Double(100, 10)
    as the configuration says, Chunk(100) and Remote(100) for comparison."""
    _full_size_properties(2, [(snn.SNN_DOUBLE, 100, 10), (snn.SNN_CHUNK, 0, 100), (snn.SNN_REMOTE, 100, 0)], 8 * 10**9, 150)


def test_config3_full_size_properties():
    """Configuration 3 (128 -> 2x512 -> 10, T = 100 000, batch 16) under its 4 GB budget: Double(316, 18)."""
    _full_size_properties(3, [(snn.SNN_DOUBLE, 316, 18), (snn.SNN_CHUNK, 0, 316)], 4 * 10**9, 1500)


def test_config4_full_size_properties():
    """Configuration 4 (1024 -> 4x8192 -> 100, T = 5000, batch 32, recurrent matrices 90 % zero) as the benchmark
    times it: Double(512, 64) under the 32 GB budget (the forward pass's currents kept, stage launches over compressed
    rows), the same intervals under the smallest budget they run in (currents recomputed, no pipelining buffers), and
    Remote(512) under the 32 GB."""
    _full_size_properties(4, [(snn.SNN_DOUBLE, 512, 64), (snn.SNN_DOUBLE, 512, 64, "min"), (snn.SNN_REMOTE, 512, 0)],
                          32 * 10**9, 5)


def test_config4_widths_short():
    """Configuration 4's layer widths (1024 -> 4 x 8192 -> 100, recurrent matrices 90 % zero with a
    per-seed mask) at a short T and small batch: 16 neurons per thread in the gather kernels, the
    streamed adjoint kernel, masked gradients."""
    w = synth.config(4, T=6, B=2)
    _full_parity(w, [(snn.SNN_STANDARD, 0, 0), (snn.SNN_DOUBLE, 4, 2)], nthreads=2, check_states=True)


@pytest.mark.parametrize("hidden,B,T,density,gain", [((1024,), 5, 30, 0.1, 1.0), ((600, 1100), 3, 24, 0.3, 0.8),
                                                     ((2048,), 3, 20, 0.1, 1.0), ((4096, 4096), 2, 10, 0.1, 1.0), ((96, 96), 4, 40, 0.2, 0.8),
                                                     ((1536,), 2, 16, 0.9, 0.5)])
def test_compressed_rows_of_masked_matrices_are_bitwise_neutral(hidden, B, T, density, gain, monkeypatch):
    """A masked recurrent matrix is also kept as compressed rows (only the synapses that exist), and the kernels
    that gather its rows walk those (recompute; from 2048 neurons also the sequential part of the forward pass).
    Adding +0.0f where no synapse exists changes nothing, so spike trains, membrane potentials -- the forward
    pass's and the recomputed ones -- and gradients must be the very bits of the dense-stored walk (SNN_CSR=0), and
    match the oracle.  Widths: one sub-range, several, a ragged last one, a row with more than 64 entries in a
    sub-range (density 0.9), and a layer narrow enough for the register-stationary kernels (which ignore the
    compressed form)."""
    w = synth.Workload("csr_" + "x".join(map(str, hidden)), 40, hidden, 6, T=T, B=B, p_in=0.1, gain=gain,
                       rec_density=density, seed=51 + B)
    d = synth.generate(w)
    L = len(hidden)
    got = {}
    # (the adjoint recurrence of wide masked layers has a kernel of its own over the compressed rows, with its own
    # order of summation: kept out of this bitwise comparison, it has a test of its own)
    monkeypatch.setenv("SNN_WS_KERNEL", "chip")
    for csr in ("1", "0"):
        monkeypatch.setenv("SNN_CSR", csr)
        net = snn.from_workload(w, d)
        try:
            net.snn_bind_inputs(d["in_spikes"], d["labels"], w.T)
            states = net.snn_debug_states(w.T)
            net.snn_bptt(snn.SNN_DOUBLE, 8, 3)
            recomputed = [net.snn_get_state(l, t) for l in range(L) for t in (1, w.T // 2, w.T)]
            got[csr] = (_gpu_grads(net, L), [net.snn_get_spikes(l, w.T) for l in range(L)], states, recomputed)
        finally:
            net.snn_destroy()
    monkeypatch.delenv("SNN_CSR")
    monkeypatch.delenv("SNN_WS_KERNEL")
    assert _identical(got["1"][0], got["0"][0])
    for a, b in zip(got["1"][1], got["0"][1]):
        assert np.array_equal(a, b) and a.sum() > 0
    assert np.array_equal(got["1"][2].view(np.uint32), got["0"][2].view(np.uint32))
    for a, b in zip(got["1"][3], got["0"][3]):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    _full_parity(w, [(snn.SNN_STANDARD, 0, 0), (snn.SNN_DOUBLE, 8, 3), (snn.SNN_CHUNK, 0, 5)], nthreads=4,
                 probe_states=[(L - 1, w.T), (0, 2)])


def test_compressed_rows_keep_denormal_sums():
    """Weights so small that every synaptic sum is a denormal number: the compressed-row walk accumulates with LDS
    add instructions, which must round and keep denormals exactly like the vector adds of the dense-stored walk
    and like the oracle.  Nobody fires (potentials around 1e-38), so the check is on the membrane potentials."""
    w = synth.Workload("csr_denormal_40-1024-6", 40, (1024,), 6, T=12, B=3, p_in=0.2, gain=1.0, rec_density=0.2, seed=77)
    d = synth.generate(w)
    d["W_in"] = [np.float32(3e-39) * np.sign(a) * (1 + np.arange(a.size, dtype=np.float32).reshape(a.shape) % 7) for a in d["W_in"]]
    d["W_rec"] = [(np.float32(1e-39) * np.sign(a) * (1 + np.arange(a.size, dtype=np.float32).reshape(a.shape) % 5)).astype(np.float32)
                  * d["rec_mask"][l] for l, a in enumerate(d["W_rec"])]
    ref = _oracle(w, d, want_v=True, backward=False, forced_spikes=None)
    assert 0 < np.abs(ref.v[0]).max() < 1e-35 and (np.abs(ref.v[0][ref.v[0] != 0]) < 1.1754944e-38).any()
    # the recurrent walk needs spikes: force a spike train through the micro-benchmark entry, then rebuild states
    hid = synth.forced_spike_trains(w, [0.1])
    ref_forced = _oracle(w, d, want_v=True, backward=False, forced_spikes=[h.astype(np.float32) for h in hid])
    net = snn.from_workload(w, d)
    try:
        net.snn_forward(d["in_spikes"], d["labels"], w.T)
        assert np.array_equal(net.snn_debug_states(w.T)[:, :, :1024].view(np.uint32), ref.v[0].view(np.uint32))
        net.snn_debug_currents(hid, 4)  # replaces the stored hidden spike train
        for t in (2, 7, 12):
            assert np.array_equal(net.snn_get_state(0, t).view(np.uint32), ref_forced.v[0][t - 1].view(np.uint32)), t
    finally:
        net.snn_destroy()


@pytest.mark.parametrize("hidden,B,T,density", [
    ((1024,), 5, 30, 0.12),       # about half of the (row, sub-range) pairs have more than 64 entries: the rest kernel
    ((2048, 600), 3, 24, 0.1),    # a ragged last sub-range and a ragged block of presynaptic rows
    ((1536,), 32, 10, 0.1),       # one whole time step per tile
    ((1024, 1024), 7, 40, 0.05),  # tiles of four steps, the last one ragged
    ((1024,), 33, 8, 0.1),        # batch above 32: dense accumulators (the choice must not change the result)
    ((1024,), 4, 12, 0.6)])       # too dense for one entry per lane: dense accumulators
def test_weight_gradients_over_compressed_rows(hidden, B, T, density, monkeypatch):
    """With the tiled event-driven weight-gradient kernel, a masked recurrent matrix accumulates its gradient per
    existing synapse, through its compressed rows (k_dw_csr + k_dw_csr_rest) instead of over the dense tile
    (SNN_DW_CSR=0).  Per synapse the sequence of operations is the same, so the gradients must be identical bit for
    bit (zero where no synapse exists), eagerly and as a replayed graph, and match the oracle under every
    strategy."""
    w = synth.Workload("dwcsr_" + "x".join(map(str, hidden)), 40, hidden, 6, T=T, B=B, p_in=0.1, gain=0.8,
                       rec_density=density, seed=91 + B)
    d = synth.generate(w)
    L = len(hidden)
    monkeypatch.setenv("SNN_DW", "tile")
    got = {}
    for mode in ("csr", "dense"):
        if mode == "dense":
            monkeypatch.setenv("SNN_DW_CSR", "0")
        else:
            monkeypatch.delenv("SNN_DW_CSR", raising=False)
        net = snn.from_workload(w, d)
        try:
            net.snn_bind_inputs(d["in_spikes"], d["labels"], w.T)
            net.snn_bptt(snn.SNN_DOUBLE, 8, 3)
            got[mode] = _gpu_grads(net, L)
            net.snn_bptt(snn.SNN_DOUBLE, 8, 3)  # the replayed graph
            assert _identical(_gpu_grads(net, L), got[mode]), mode
            net.snn_bptt(snn.SNN_STANDARD, 0, 0)
            assert _identical(_gpu_grads(net, L), got[mode]), mode
        finally:
            net.snn_destroy()
    monkeypatch.delenv("SNN_DW_CSR", raising=False)
    assert _identical(got["csr"], got["dense"])
    for l in range(L):
        assert np.all(got["csr"][1][l][d["rec_mask"][l] == 0] == 0.0) and np.abs(got["csr"][1][l]).max() > 0
    _full_parity(w, [(snn.SNN_STANDARD, 0, 0), (snn.SNN_DOUBLE, 8, 3), (snn.SNN_CHUNK, 0, 5)], nthreads=4)
    monkeypatch.delenv("SNN_DW")


@pytest.mark.parametrize("hidden,B,T,density,window", [
    ((2048,), 5, 14, 0.1, 0.0),        # one job, a ragged batch group (5 = 4 + 1)
    ((1536, 1100), 3, 12, 0.3, 0.0),   # two jobs of different widths in one launch, ragged row blocks
    ((4096, 4096), 8, 10, 0.1, 0.0),   # two batch groups
    ((2048,), 2, 9, 0.9, 0.0),         # rows of ~1840 entries: more than one pass of 14 x 64
    ((2048, 256), 6, 12, 0.2, 0.0),    # a narrow layer beside it (weights in registers)
    ((3072,), 4, 10, 0.15, 0.5)])      # under a surrogate window, forced (the library would list rows)
def test_chip_wide_adjoint_over_compressed_rows(hidden, B, T, density, window, monkeypatch):
    """Wide layers (more than 1024 neurons) with a masked recurrent matrix run the adjoint recurrence chip-wide over
    the compressed rows: four batch elements per workgroup with their dv_{t+1} in LDS, rows dealt to wavefronts,
    a barrier per batch group and step.  A row is summed in the order of the rows kernel (lane-strided, two
    accumulators, butterfly), so the gradients must be the very bits of that kernel evaluating every row
    (SNN_WS_KERNEL=rows_all); they must agree with the dense-stored chip-wide kernel (SNN_CSR=0) within the gradient
    tolerance, and match the oracle under every strategy."""
    w = synth.Workload("csrw_" + "x".join(map(str, hidden)), 40, hidden, 6, T=T, B=B, p_in=0.1, gain=0.8,
                       rec_density=density, seed=71 + B)
    d = synth.generate(w)
    L = len(hidden)
    got = {}
    for mode in ("csrw", "rows_all", "dense"):
        monkeypatch.delenv("SNN_WS_KERNEL", raising=False)
        monkeypatch.delenv("SNN_CSR", raising=False)
        if mode == "rows_all":
            monkeypatch.setenv("SNN_WS_KERNEL", "rows_all")
        elif mode == "dense":
            monkeypatch.setenv("SNN_CSR", "0")
            monkeypatch.setenv("SNN_WS_KERNEL", "chip")
        elif window > 0:
            monkeypatch.setenv("SNN_WS_KERNEL", "csrw")
        net = snn.from_workload(w, d, surr_window=window)
        try:
            net.snn_bind_inputs(d["in_spikes"], d["labels"], w.T)
            net.snn_bptt(snn.SNN_DOUBLE, 8, 3)
            got[mode] = _gpu_grads(net, L)
            net.snn_bptt(snn.SNN_DOUBLE, 8, 3)  # the replayed graph
            assert _identical(_gpu_grads(net, L), got[mode]), mode
        finally:
            net.snn_destroy()
    monkeypatch.delenv("SNN_WS_KERNEL", raising=False)
    monkeypatch.delenv("SNN_CSR", raising=False)
    assert _identical(got["csrw"], got["rows_all"])
    flat = lambda g: list(g[0]) + list(g[1]) + [g[2]]
    for a, b in zip(flat(got["csrw"]), flat(got["dense"])):
        scale = float(np.max(np.abs(b))) or 1.0
        assert float(np.max(np.abs(a - b))) <= 1e-4 * scale
    if window <= 0:
        _full_parity(w, [(snn.SNN_STANDARD, 0, 0), (snn.SNN_DOUBLE, 8, 3), (snn.SNN_CHUNK, 0, 5)], nthreads=4)


@pytest.mark.parametrize("hidden,B,T,density,window", [((1088,), 5, 14, 1.0, 0.4), ((2048, 1100), 3, 12, 0.15, 0.5),
                                                      ((300, 1026), 4, 10, 1.0, 0.3)])
def test_event_driven_adjoint_under_the_surrogate_window(hidden, B, T, density, window, monkeypatch):
    """With a surrogate window only the neurons whose potential is inside it have a non-zero spike derivative; the
    adjoint kernel for wide layers under a window lists those neurons from the stored potentials (ballot + popcount
    prefix) and evaluates only their rows of W_rec . dv -- compressed rows for a masked matrix.  Checked: against
    the oracle with the same window; bit-identical to the same kernel evaluating every row (SNN_WS_KERNEL=rows_all);
    within the gradient tolerance of the chip-wide kernels with the same window (SNN_WS_KERNEL=chip); and the list
    really is short (the fraction of neurons inside the window is printed)."""
    w = synth.Workload("win_rows_" + "x".join(map(str, hidden)), 40, hidden, 6, T=T, B=B, p_in=0.1, gain=0.7,
                       rec_density=density, seed=61 + B)
    d = synth.generate(w)
    L = len(hidden)
    got = {}
    for mode in ("rows", "rows_all", "chip", None):
        if mode is None:
            monkeypatch.delenv("SNN_WS_KERNEL", raising=False)
        else:
            monkeypatch.setenv("SNN_WS_KERNEL", mode)
        net = snn.from_workload(w, d, surr_window=window)
        try:
            net.snn_bind_inputs(d["in_spikes"], d["labels"], w.T)
            net.snn_bptt(snn.SNN_DOUBLE, 8, 3)
            got[mode] = _gpu_grads(net, L)
        finally:
            net.snn_destroy()
    monkeypatch.delenv("SNN_WS_KERNEL", raising=False)
    assert _identical(got["rows"], got["rows_all"])
    flat = lambda g: list(g[0]) + list(g[1]) + [g[2]]
    for a, b in zip(flat(got["rows"]), flat(got["chip"])):
        scale = float(np.max(np.abs(b))) or 1.0
        assert float(np.max(np.abs(a - b))) <= 1e-4 * scale
    if max(hidden) > 1024 and min(hidden) > 1024:
        assert _identical(got[None], got["rows"])  # the library's own choice for wide layers under a window
    first, ref = _full_parity(w, [(snn.SNN_STANDARD, 0, 0), (snn.SNN_DOUBLE, 8, 3), (snn.SNN_CHUNK, 0, 5)], nthreads=4,
                              window=window)
    inside = [float((np.abs(v - w.theta) < window).mean()) for v in ref.v]
    print(f"[{w.name}] fraction of (t, b, neuron) inside the window of {window}: {[round(x, 4) for x in inside]}")
    assert all(0.0 < x < 0.5 for x in inside)


@pytest.mark.parametrize("hidden,B,T,tier_env,strategies", [
    ((256, 256), 4, 3000, "direct", [(2, 100, 0), (3, 200, 20)]),
    ((200, 300), 3, 2600, "dma", [(3, 150, 30), (2, 64, 0)]),
    ((1088,), 2, 2000, "dma", [(3, 60, 12)])])
def test_spike_bitmasks_on_the_host_tier(hidden, B, T, tier_env, strategies, monkeypatch):
    """spike_tier 1: under Remote and Double the hidden layers' spike bitmasks of finished coarse segments travel to
    pinned host memory and come back before the segment is recomputed; HBM keeps a ring of 2 C + 1600 steps of them.
    Gradients must be the very bits of the run that keeps every bitmask in HBM (eager and as a replayed graph, with
    the states on either host tier), the HBM spike bytes must be the ring's, snn_bytes_required must drop by the
    difference, the accessors must still return the whole spike train and every state, and all of it must match the
    oracle."""
    monkeypatch.setenv("SNN_HOST_TIER", tier_env)
    w = synth.Workload("spk_host_" + "x".join(map(str, hidden)), 60, hidden, 6, T=T, B=B, p_in=0.05, gain=0.5, seed=71 + B)
    d = synth.generate(w)
    L = len(hidden)
    ref_net = snn.from_workload(w, d)
    net = snn.from_workload(w, d, spike_tier=1)
    try:
        ref_net.snn_bind_inputs(d["in_spikes"], d["labels"], w.T)
        net.snn_bind_inputs(d["in_spikes"], d["labels"], w.T)
        for strat, C, F in strategies:
            st0 = ref_net.snn_bptt(strat, C, F)
            ref = _gpu_grads(ref_net, L)
            st1 = net.snn_bptt(strat, C, F)
            assert _identical(_gpu_grads(net, L), ref), (strat, C, F, "eager")
            ring = 2 * C + 1600
            words = sum(-(-n // 64) for n in hidden)
            assert st0.bytes_spikes - st1.bytes_spikes == (w.T + 1 - ring) * w.B * words * 8
            assert st1.bytes_host_spikes == (w.T + 1) * w.B * words * 8 and st0.bytes_host_spikes == 0
            assert st1.spike_d2h_bytes == w.T * w.B * words * 8 and st1.spike_h2d_bytes >= st1.spike_d2h_bytes
            assert np.allclose(list(st1.firing_rate)[:L], list(st0.firing_rate)[:L], atol=1e-7)
            need0 = snn.snn_bytes_required(ref_net.cfg, strat, w.T, C, F)
            need1 = snn.snn_bytes_required(net.cfg, strat, w.T, C, F)
            assert need0 - need1 == (w.T + 1 - ring) * w.B * words * 8
            st2 = net.snn_bptt(strat, C, F, need1)  # runs inside the smaller budget
            assert _identical(_gpu_grads(net, L), ref), (strat, C, F, "tight budget")
            assert st2.bytes_states + st2.bytes_spikes + st2.bytes_workspace == need1
            for rep in range(2):
                net.snn_bptt(strat, C, F, want_stats=False)
                assert _identical(_gpu_grads(net, L), ref), (strat, C, F, "graph", rep)
            for l in range(L):  # the whole spike train comes back from the host for the accessors
                assert np.array_equal(net.snn_get_spikes(l, w.T), ref_net.snn_get_spikes(l, w.T))
            assert np.array_equal(net.snn_get_state(L - 1, w.T), ref_net.snn_get_state(L - 1, w.T))
        # strategies without a host tier ignore the setting
        net.snn_bptt(snn.SNN_CHUNK, 0, 50)
        ref_net.snn_bptt(snn.SNN_CHUNK, 0, 50)
        assert _identical(_gpu_grads(net, L), _gpu_grads(ref_net, L))
    finally:
        net.snn_destroy()
        ref_net.snn_destroy()
    monkeypatch.delenv("SNN_HOST_TIER")
    short = synth.Workload(w.name + "_oracle", 60, hidden, 6, T=T, B=B, p_in=0.05, gain=0.5, seed=71 + B)
    strat, C, F = strategies[0]
    dd = synth.generate(short)
    ref32 = _oracle(short, dd, want_v=True, nthreads=4, backward=False)
    ref64 = _oracle_f64_on_f32_trajectory(short, dd, ref32, 4)
    net = snn.from_workload(short, dd, spike_tier=1)
    try:
        net.snn_bind_inputs(dd["in_spikes"], dd["labels"], short.T)
        net.snn_bptt(strat, C, F)
        assert _check_spikes(net, short, ref32, short.name) == 0
        _check_grads(_gpu_grads(net, L), ref64, short.name)
    finally:
        net.snn_destroy()


def test_spike_ring_with_the_compressed_row_kernels(monkeypatch):
    """The kernels that walk compressed rows or stage their own operands address the stored spike words through the
    ring when spike_tier = 1 keeps only 2 C + 1600 steps of them in HBM: forward and recompute gathers over compressed
    rows, the chip-wide adjoint, the tiled and the per-synapse weight-gradient kernels (forced for this small matrix).
    Gradients, spike trains and a recomputed state must be the very bits of the run that keeps every bitmask in HBM."""
    monkeypatch.setenv("SNN_HOST_TIER", "dma")
    monkeypatch.setenv("SNN_DW", "tile")
    monkeypatch.setenv("SNN_CSR", "1")
    w = synth.Workload("spk_ring_csr_2048", 60, (2048,), 6, T=1800, B=3, p_in=0.05, gain=0.6, rec_density=0.1, seed=97)
    d = synth.generate(w)
    ref_net = snn.from_workload(w, d)
    net = snn.from_workload(w, d, spike_tier=1)
    try:
        ref_net.snn_bind_inputs(d["in_spikes"], d["labels"], w.T)
        net.snn_bind_inputs(d["in_spikes"], d["labels"], w.T)
        for strat, C, F in [(snn.SNN_DOUBLE, 40, 10), (snn.SNN_REMOTE, 64, 0)]:
            st0 = ref_net.snn_bptt(strat, C, F)
            st1 = net.snn_bptt(strat, C, F)
            assert st1.bytes_spikes < st0.bytes_spikes and st1.bytes_host_spikes > 0
            assert _identical(_gpu_grads(net, 1), _gpu_grads(ref_net, 1)), (strat, "eager")
            net.snn_bptt(strat, C, F, want_stats=False)
            assert _identical(_gpu_grads(net, 1), _gpu_grads(ref_net, 1)), (strat, "graph")
        g = _gpu_grads(net, 1)
        assert np.abs(g[1][0]).max() > 0 and np.all(g[1][0][d["rec_mask"][0] == 0] == 0.0)
        assert np.array_equal(net.snn_get_spikes(0, w.T), ref_net.snn_get_spikes(0, w.T))
        assert np.array_equal(net.snn_get_state(0, 901).view(np.uint32), ref_net.snn_get_state(0, 901).view(np.uint32))
    finally:
        net.snn_destroy()
        ref_net.snn_destroy()
    for k in ("SNN_HOST_TIER", "SNN_DW", "SNN_CSR"):
        monkeypatch.delenv(k)


@pytest.mark.parametrize("n_in,hidden,n_out,B,T", [(70, (100, 72, 130), 7, 3, 40), (50, (300, 1026), 5, 12, 21),
                                                   (40, (256, 256), 20, 32, 70), (33, (520,), 9, 64, 9),
                                                   (33, (130, 64), 3, 40, 17), (24, (64,), 2, 1, 30)])
def test_event_driven_tiled_weight_gradients(n_in, hidden, n_out, B, T, monkeypatch):
    """The tiled event-driven weight-gradient kernel (the default for networks with very large matrices, forced
    here with SNN_DW=tile): row and column tiles that are ragged, column offsets that are not multiples of four,
    batches that fill a 64-row tile exactly, partly, and with one element, several time steps per tile.  Against the
    oracle, bit-identical between strategies, and bit-identical to the matrix-core contraction."""
    w = synth.Workload("dwtile_" + "x".join(map(str, hidden)), n_in, hidden, n_out, T=T, B=B, p_in=0.1, gain=0.5, seed=81 + B)
    d = synth.generate(w)
    L = len(hidden)
    got = {}
    for mode in ("tile", "mfma"):
        monkeypatch.setenv("SNN_DW", mode)
        net = snn.from_workload(w, d)
        try:
            net.snn_bind_inputs(d["in_spikes"], d["labels"], w.T)
            net.snn_bptt(snn.SNN_CHUNK, 0, 6)
            got[mode] = _gpu_grads(net, L)
        finally:
            net.snn_destroy()
    flat = lambda g: list(g[0]) + list(g[1]) + [g[2]]
    for a, b in zip(flat(got["tile"]), flat(got["mfma"])):
        assert np.array_equal(a, b)  # the library picks between the two from the firing rates, step by step
    monkeypatch.setenv("SNN_DW", "tile")
    first, _ = _full_parity(w, [(snn.SNN_STANDARD, 0, 0), (snn.SNN_CHUNK, 0, 6), (snn.SNN_DOUBLE, 8, 3), (snn.SNN_REMOTE, 5, 0)],
                            nthreads=4, check_states=False)
    assert _identical(first, got["tile"])
    monkeypatch.delenv("SNN_DW")
