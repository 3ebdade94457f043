"""Pins for the CPU oracle: everything here checks the oracle against something
other than itself -- a hand-computed trace, closed forms, finite differences,
an automatic-differentiation library, the paper's memory/time formulas and the
execution order drawn in its Fig. 1.  None of these tests needs a GPU."""
import os

import numpy as np
import pytest

import oracle
import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _parse(path):
    out = {}
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, rest = line.split(None, 1)
        rows = [[float(x) for x in r.split()] for r in rest.split("/")]
        out[key] = np.array(rows)
    return out


def _tiny(seed, n_in=5, hidden=(6, 4), n_out=3, T=7, B=2, p=0.3, scale=0.7):
    rng = np.random.default_rng(seed)
    pre = [n_in] + list(hidden[:-1])
    W_in = [rng.standard_normal((pre[l], n)) * scale for l, n in enumerate(hidden)]
    W_rec = [rng.standard_normal((n, n)) * scale for n in hidden]
    W_out = rng.standard_normal((hidden[-1], n_out)) * scale
    x = (rng.random((T, B, n_in)) < p).astype(np.uint8)
    y = rng.integers(0, n_out, B).astype(np.int32)
    return dict(n_in=n_in, n_hidden=list(hidden), n_out=n_out, W_in=W_in, W_rec=W_rec, W_out=W_out,
                in_spikes=x, labels=y)


def _run(net, **kw):
    return oracle.bptt(net["n_in"], net["n_hidden"], net["n_out"], net["W_in"], net["W_rec"],
                       net["W_out"], net["in_spikes"], net["labels"], **kw)


# --------------------------------------------------------------------------- forward

@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_hand_trace(dtype):
    """3-neuron, 5-step membrane trace computed by hand (tests/golden/hand_trace_3neuron.txt)."""
    g = _parse(os.path.join(GOLD, "hand_trace_3neuron.txt"))
    x = g["x"].astype(np.uint8)[:, None, :]
    r = oracle.bptt(2, [3], 2, [g["W_in"]], [g["W_rec"]], g["W_out"], x, [0], alpha=0.5, beta=0.5,
                    theta=1.0, dtype=dtype, want_v=True)
    assert np.array_equal(r.v[0][:, 0, :], g["v"].astype(dtype))          # dyadic: exact
    assert np.array_equal(r.spikes[0][:, 0, :], g["s"].astype(dtype))
    # u_t is not returned; its time average is
    assert np.allclose(r.ubar[0], g["u"].mean(axis=0), rtol=0, atol=1e-6)
    assert np.allclose(r.ubar[0], g["ubar"][0], rtol=0, atol=1e-6)
    assert abs(r.loss - g["loss"][0, 0]) < 2e-6
    assert np.allclose(r.dW_out, g["dW_out"], rtol=0, atol=2e-6)


def test_threshold_is_strict():
    """v == theta exactly does not fire (convention: s = 1 iff v > theta)."""
    x = np.array([1, 0, 1], dtype=np.uint8).reshape(3, 1, 1)
    r = oracle.bptt(1, [1], 1, [np.array([[1.0]])], [np.array([[0.0]])], np.array([[1.0]]), x, [0],
                    alpha=0.5, dtype=np.float32, want_v=True)
    assert r.v[0][:, 0, 0].tolist() == [1.0, 0.5, 1.25]
    assert r.spikes[0][:, 0, 0].tolist() == [0.0, 0.0, 1.0]


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_leaky_integrator_closed_form(dtype):
    """With a threshold nobody reaches, every neuron is a leaky integrator:
    v_t = sum_{k<=t} alpha^(t-k) * (W_in^T x_k)  (geometric sum, textbook closed form)."""
    net = _tiny(3, hidden=(6,), T=9)
    alpha = 0.8
    r = _run(net, alpha=alpha, theta=1e6, dtype=np.float64, want_v=True, backward=False)
    cur = np.einsum("tbj,jn->tbn", net["in_spikes"].astype(np.float64), net["W_in"][0])
    T = cur.shape[0]
    expect = np.zeros_like(cur)
    for t in range(T):
        for k in range(t + 1):
            expect[t] += alpha ** (t - k) * cur[k]
    assert np.allclose(r.v[0], expect, rtol=1e-12, atol=1e-12)
    assert not np.any(r.spikes[0])
    # the readout never sees a spike: ubar = 0 and the loss is ln(n_out)
    assert np.all(r.ubar == 0)
    assert abs(r.loss - np.log(net["n_out"])) < 1e-12


def test_loss_is_log_nout_when_readout_weights_vanish():
    net = _tiny(4)
    net["W_out"] = np.zeros_like(net["W_out"])
    r = _run(net, dtype=np.float64)
    assert abs(r.loss - np.log(net["n_out"])) < 1e-12
    # nothing but W_out can get a gradient then (ds of the last layer is W_out . du = 0)
    assert all(np.all(d == 0) for d in r.dW_in + r.dW_rec)
    # softmax - onehot sums to zero over the classes, so each dW_out row sums to zero
    assert np.allclose(r.dW_out.sum(axis=1), 0, atol=1e-15)
    assert np.any(r.dW_out != 0)


def test_reset_and_recurrence_single_neuron():
    """One neuron, constant drive 0.6 per step, alpha = 1, self-weight w: closed form by hand.
    v: 0.6, 1.2 (spike), 1.2 - 1 + 0.6 + w, ...  with w = -0.25: 0.6, 1.2*, 0.55, 1.15*, 0.5."""
    x = np.ones((5, 1, 1), dtype=np.uint8)
    r = oracle.bptt(1, [1], 1, [np.array([[0.6]])], [np.array([[-0.25]])], np.array([[1.0]]), x, [0],
                    alpha=1.0, dtype=np.float64, want_v=True, backward=False)
    assert np.allclose(r.v[0][:, 0, 0], [0.6, 1.2, 0.55, 1.15, 0.5], atol=1e-15)
    assert r.spikes[0][:, 0, 0].tolist() == [0, 1, 0, 1, 0]


# --------------------------------------------------------------------------- backward

def _flat(net):
    return np.concatenate([w.ravel() for w in net["W_in"]] + [w.ravel() for w in net["W_rec"]] +
                          [net["W_out"].ravel()])


def _unflat(net, vec):
    out = dict(net)
    pos = 0
    for key in ("W_in", "W_rec"):
        lst = []
        for w in net[key]:
            lst.append(vec[pos:pos + w.size].reshape(w.shape))
            pos += w.size
        out[key] = lst
    out["W_out"] = vec[pos:pos + net["W_out"].size].reshape(net["W_out"].shape)
    return out


@pytest.mark.parametrize("seed,hidden", [(0, (6, 4)), (1, (5,)), (2, (3, 4, 3))])
def test_backward_matches_finite_differences(seed, hidden):
    """Heaviside replaced by S(x) = x/(1+k|x|) (derivative = the surrogate): the network is
    smooth and the analytic gradient must equal central differences, for every tensor."""
    net = _tiny(seed, hidden=hidden, T=6, scale=0.5)
    kw = dict(mode=oracle.SMOOTH, dtype=np.float64, alpha=0.9, beta=0.8, surr_beta=3.0)
    r = _run(net, **kw)
    ana = np.concatenate([d.ravel() for d in r.dW_in] + [d.ravel() for d in r.dW_rec] + [r.dW_out.ravel()])
    w0 = _flat(net)
    rng = np.random.default_rng(seed)
    idx = rng.choice(w0.size, size=min(60, w0.size), replace=False)
    h = 1e-6
    for i in idx:
        wp, wm = w0.copy(), w0.copy()
        wp[i] += h
        wm[i] -= h
        lp = _run(_unflat(net, wp), backward=False, **kw).loss
        lm = _run(_unflat(net, wm), backward=False, **kw).loss
        fd = (lp - lm) / (2 * h)
        assert abs(fd - ana[i]) <= 1e-7 * max(1.0, np.abs(ana).max()) + 1e-9, (i, fd, ana[i])


def _autograd_reference(net, alpha, beta, theta, k, window):
    """Heaviside forward written with torch ops, the surrogate (cut to zero outside ``window``
    when that is positive) as the backward of the threshold; torch derives everything else."""
    import torch

    class Spike(torch.autograd.Function):
        @staticmethod
        def forward(ctx, x):
            ctx.save_for_backward(x)
            return (x > 0).to(x.dtype)

        @staticmethod
        def backward(ctx, go):
            (x,) = ctx.saved_tensors
            g = go / (1 + k * x.abs()) ** 2
            if window > 0:
                g = torch.where(x.abs().to(torch.float32) < torch.tensor(window, dtype=torch.float32),
                                g, torch.zeros_like(g))
            return g

    Wi = [torch.tensor(w, dtype=torch.float64, requires_grad=True) for w in net["W_in"]]
    Wr = [torch.tensor(w, dtype=torch.float64, requires_grad=True) for w in net["W_rec"]]
    Wo = torch.tensor(net["W_out"], dtype=torch.float64, requires_grad=True)
    x = torch.tensor(net["in_spikes"], dtype=torch.float64)
    T, B, _ = x.shape
    v = [torch.zeros(B, n, dtype=torch.float64) for n in net["n_hidden"]]
    s = [torch.zeros(B, n, dtype=torch.float64) for n in net["n_hidden"]]
    u = torch.zeros(B, net["n_out"], dtype=torch.float64)
    usum = torch.zeros_like(u)
    spikes, inside = [], 0
    for t in range(T):
        below = x[t]
        for l in range(len(v)):
            v[l] = alpha * v[l] - theta * s[l] + below @ Wi[l] + s[l] @ Wr[l]
            s[l] = Spike.apply(v[l] - theta)
            inside += int(((v[l] - theta).abs() < window).sum()) if window > 0 else 0
            below = s[l]
        spikes.append([q.detach().numpy().copy() for q in s])
        u = beta * u + s[-1] @ Wo
        usum = usum + u
    loss = torch.nn.functional.cross_entropy(usum / T, torch.tensor(net["labels"], dtype=torch.long))
    loss.backward()
    return spikes, loss.item(), [w.grad.numpy() for w in Wi + Wr + [Wo]], inside


@pytest.mark.parametrize("window", [0.0, 0.4])
def test_backward_matches_autograd_with_surrogate(window):
    """Heaviside forward with the surrogate derivative in the backward pass, against torch's
    reverse-mode differentiation of an independently written forward (double precision).  The
    backward equations of the oracle are hand-derived; here a library derives them.  With a
    window the surrogate is zero wherever |v - theta| >= window."""
    pytest.importorskip("torch")
    net = _tiny(7, n_in=6, hidden=(7, 5), n_out=4, T=9, B=3, scale=0.8)
    alpha, beta, theta, k = 0.9, 0.85, 1.0, 10.0
    spikes, loss, grads, inside = _autograd_reference(net, alpha, beta, theta, k, window)

    r = _run(net, dtype=np.float64, alpha=alpha, beta=beta, theta=theta, surr_beta=k, surr_window=window)
    for l in range(len(net["n_hidden"])):
        assert np.array_equal(r.spikes[l], np.stack([sp[l] for sp in spikes]))
    assert abs(r.loss - loss) < 1e-12
    for mine, ref in zip(r.dW_in + r.dW_rec + [r.dW_out], grads):
        assert np.allclose(mine, ref, rtol=1e-9, atol=1e-12)
    assert any(np.abs(d).max() > 1e-6 for d in r.dW_rec)
    if window > 0:  # the window must cut some neurons and keep others, else this case pins nothing
        total = 9 * 3 * (7 + 5)
        assert 0 < inside < total
        full = _run(net, dtype=np.float64, alpha=alpha, beta=beta, theta=theta, surr_beta=k)
        assert not np.allclose(full.dW_rec[0], r.dW_rec[0], rtol=1e-3, atol=0)


def test_surrogate_window_limits():
    """A window wider than any |v - theta| changes nothing, bit for bit; a window that admits no
    neuron leaves only the readout gradient (dW_out does not pass through any threshold), and
    the strategies still agree bit for bit with a window in force."""
    net = _tiny(11, n_in=8, hidden=(9, 6), n_out=3, T=14, B=2, scale=0.9)
    for dt in (np.float32, np.float64):
        base = _run(net, dtype=dt, want_v=True)
        vmax = max(np.abs(v - 1.0).max() for v in base.v)
        wide = _run(net, dtype=dt, surr_window=float(vmax) * 2 + 1)
        none = _run(net, dtype=dt, surr_window=1e-30)
        for a, b in zip(base.dW_in + base.dW_rec + [base.dW_out], wide.dW_in + wide.dW_rec + [wide.dW_out]):
            assert np.array_equal(a, b)
        assert np.array_equal(none.dW_out, base.dW_out) and np.abs(base.dW_out).max() > 0
        for d in none.dW_in + none.dW_rec:
            assert not d.any()
        mid = _run(net, dtype=dt, surr_window=0.5)
        assert any(not np.array_equal(a, b) for a, b in zip(mid.dW_rec, base.dW_rec))
        for strat, c, f in ((oracle.CHUNK, 0, 4), (oracle.REMOTE, 5, 0), (oracle.DOUBLE, 6, 2)):
            o = _run(net, dtype=dt, surr_window=0.5, strategy=strat, coarse=c, fine=f)
            for a, b in zip(mid.dW_in + mid.dW_rec + [mid.dW_out], o.dW_in + o.dW_rec + [o.dW_out]):
                assert np.array_equal(a, b)
    with pytest.raises(Exception):
        _run(net, dtype=np.float64, mode=oracle.SMOOTH, surr_window=0.5)


def test_masked_recurrent_gradient():
    """Gradient exists only on synapses that exist: with a recurrent mask, the result is the
    dense gradient at the masked weights, times the mask (finite differences on kept synapses)."""
    net = _tiny(11, hidden=(6,), T=6, scale=0.6)
    rng = np.random.default_rng(5)
    mask = (rng.random((6, 6)) < 0.4).astype(np.uint8)
    net["W_rec"] = [net["W_rec"][0] * mask]
    kw = dict(mode=oracle.SMOOTH, dtype=np.float64, surr_beta=3.0)
    r = _run(net, rec_mask=[mask], **kw)
    dense = _run(net, **kw)
    assert np.array_equal(r.dW_rec[0], dense.dW_rec[0] * mask)
    assert np.all(r.dW_rec[0][mask == 0] == 0)
    h = 1e-6
    for (j, i) in zip(*np.nonzero(mask)):
        wp = net["W_rec"][0].copy(); wp[j, i] += h
        wm = net["W_rec"][0].copy(); wm[j, i] -= h
        lp = _run(dict(net, W_rec=[wp]), backward=False, **kw).loss
        lm = _run(dict(net, W_rec=[wm]), backward=False, **kw).loss
        assert abs((lp - lm) / (2 * h) - r.dW_rec[0][j, i]) < 1e-7


# --------------------------------------------------------------------------- strategies

STRATS = [(oracle.STANDARD, 0, 0), (oracle.CHUNK, 0, 10), (oracle.CHUNK, 0, 7), (oracle.CHUNK, 0, 1),
          (oracle.CHUNK, 0, 50), (oracle.REMOTE, 10, 0), (oracle.REMOTE, 13, 0), (oracle.REMOTE, 50, 0),
          (oracle.DOUBLE, 20, 5), (oracle.DOUBLE, 17, 4), (oracle.DOUBLE, 50, 7), (oracle.DOUBLE, 6, 6),
          (oracle.DOUBLE, 9, 1), (oracle.HIER, 2, 5), (oracle.HIER, 3, 7), (oracle.HIER, 1, 10), (oracle.HIER, 20, 4),
          (oracle.HIER, 4, 50)]


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_all_strategies_bit_identical_to_full_storage(dtype):
    """Checkpointing changes what is stored, not what is computed: gradients, spikes and loss
    of every strategy equal those of full storage bit for bit (configuration 0)."""
    w = synth.config(0)
    d = synth.generate(w)
    args = (w.n_in, list(w.n_hidden), w.n_out, d["W_in"], d["W_rec"], d["W_out"], d["in_spikes"], d["labels"])
    ref = oracle.bptt(*args, dtype=dtype)
    assert np.abs(ref.dW_rec[0]).max() > 0
    for s, c, f in STRATS[1:]:
        r = oracle.bptt(*args, dtype=dtype, strategy=s, coarse=c, fine=f)
        assert r.loss == ref.loss
        assert np.array_equal(r.spikes[0], ref.spikes[0])
        for a, b in zip(r.dW_in + r.dW_rec + [r.dW_out], ref.dW_in + ref.dW_rec + [ref.dW_out]):
            assert np.array_equal(a, b), (s, c, f)


def test_two_layer_strategies_bit_identical():
    net = _tiny(21, n_in=12, hidden=(16, 9), n_out=5, T=37, B=3, p=0.2, scale=0.6)
    ref = _run(net, dtype=np.float32)
    for s, c, f in [(oracle.CHUNK, 0, 6), (oracle.REMOTE, 8, 0), (oracle.DOUBLE, 12, 5), (oracle.DOUBLE, 37, 6)]:
        r = _run(net, dtype=np.float32, strategy=s, coarse=c, fine=f)
        for a, b in zip(r.dW_in + r.dW_rec + [r.dW_out], ref.dW_in + ref.dW_rec + [ref.dW_out]):
            assert np.array_equal(a, b)


def test_forced_spikes_reproduce_states_and_gradients():
    """Recomputing from stored spikes (no thresholding) gives the same states: feeding the
    oracle its own spike trains reproduces v and the gradients exactly."""
    net = _tiny(22, n_in=10, hidden=(12, 8), T=20, B=2, p=0.25, scale=0.6)
    a = _run(net, dtype=np.float32, want_v=True)
    b = _run(net, dtype=np.float32, want_v=True, forced_spikes=a.spikes)
    for l in range(2):
        assert np.array_equal(a.v[l], b.v[l])
    for p, q in zip(a.dW_in + a.dW_rec, b.dW_in + b.dW_rec):
        assert np.array_equal(p, q)


def test_fig1_double_schedule_order():
    """Execution order of the Double panel of Fig. 1 (tests/golden/fig1_double_schedule.txt)."""
    gold = []
    for line in open(os.path.join(GOLD, "fig1_double_schedule.txt")):
        line = line.strip()
        if line and not line.startswith("#"):
            p = line.split()
            gold.append((p[0], int(p[1]), int(p[2]) if len(p) > 2 else 0))
    net = _tiny(5, T=11, B=1)
    r = _run(net, strategy=oracle.DOUBLE, coarse=6, fine=3, want_events=True)
    back = [e for e in r.events if e[0] != "SAVE_REMOTE"]
    assert back == gold
    assert [e for e in r.events if e[0] == "SAVE_REMOTE"] == [("SAVE_REMOTE", 0, 0), ("SAVE_REMOTE", 6, 0)]


def test_fig1_chunk_and_remote_order():
    """Fig. 1, middle panels: checkpoints every 3rd state (x_0, x_3, x_6, x_9 of x_0..x_11),
    each chunk recomputed (blue) then back-propagated (red), right to left; Remote loads
    the checkpoint first."""
    net = _tiny(5, T=11, B=1)
    r = _run(net, strategy=oracle.CHUNK, fine=3, want_events=True)
    assert [e for e in r.events if e[0] == "SAVE_LOCAL"] == [("SAVE_LOCAL", c, 0) for c in (0, 3, 6, 9)]
    assert [e for e in r.events if e[0] != "SAVE_LOCAL"] == [
        ("REFWD2", 9, 11), ("BACKWARD", 11, 10), ("REFWD2", 6, 9), ("BACKWARD", 9, 7),
        ("REFWD2", 3, 6), ("BACKWARD", 6, 4), ("REFWD2", 0, 3), ("BACKWARD", 3, 1)]
    r = _run(net, strategy=oracle.REMOTE, coarse=3, want_events=True)
    assert [e for e in r.events if e[0] not in ("SAVE_REMOTE",)] == [
        ("LOAD_REMOTE", 9, 0), ("REFWD2", 9, 11), ("BACKWARD", 11, 10),
        ("LOAD_REMOTE", 6, 0), ("REFWD2", 6, 9), ("BACKWARD", 9, 7),
        ("LOAD_REMOTE", 3, 0), ("REFWD2", 3, 6), ("BACKWARD", 6, 4),
        ("LOAD_REMOTE", 0, 0), ("REFWD2", 0, 3), ("BACKWARD", 3, 1)]


@pytest.mark.parametrize("T,C,F", [(64, 16, 4), (4096 // 16, 64, 8), (100, 25, 5)])
def test_memory_and_time_closed_forms(T, C, F):
    """State slots and pass counts against the paper's closed forms (divisible case, which is
    what the paper assumes): M_Base = T, M_Standard = chunk + T/chunk, M_Remote = chunk + 1,
    M_Double = chunk + remote_chunk/chunk; T_Standard has one recompute pass, T_Double two;
    N_c = 2 T / remote_chunk transfers."""
    net = _tiny(9, T=T, B=1, hidden=(4,))
    st = _run(net, strategy=oracle.STANDARD).stats
    assert st["local_slots"] == T and st["refwd1_steps"] == st["refwd2_steps"] == 0
    st = _run(net, strategy=oracle.CHUNK, fine=F).stats
    assert st["local_slots"] == F + T // F
    assert (st["fwd_steps"], st["refwd2_steps"], st["bwd_steps"]) == (T, T, T)
    st = _run(net, strategy=oracle.REMOTE, coarse=C).stats
    assert st["local_slots"] == C + 1 and st["remote_slots"] == T // C
    assert st["remote_writes"] + st["remote_reads"] == 2 * (T // C)
    assert (st["fwd_steps"], st["refwd2_steps"], st["bwd_steps"]) == (T, T, T)
    st = _run(net, strategy=oracle.DOUBLE, coarse=C, fine=F).stats
    assert st["local_slots"] == F + C // F
    assert st["remote_writes"] + st["remote_reads"] == 2 * (T // C)
    assert (st["fwd_steps"], st["refwd2_steps"], st["bwd_steps"]) == (T, T, T)
    # the extra pass stops at the last fine checkpoint of each coarse segment
    assert st["refwd1_steps"] == (T // C) * (C - F)


@pytest.mark.parametrize("T,F,NL", [(64, 4, 4), (100, 5, 2), (96, 8, 3), (60, 6, 10)])
def test_hierarchical_closed_forms(T, F, NL):
    """Section "Hierarchical Checkpointing": M_Hier = chunk + nb_local states in local memory; checkpoints
    travel in batches of nb_local, the last batch never leaves local memory, so there are
    nb_checkpoints/nb_local - 1 batch writes and as many batch reads (the reading of N_c that the
    paper's prose gives); one recompute pass as in Standard Checkpointing."""
    net = _tiny(9, T=T, B=1, hidden=(4,))
    st = _run(net, strategy=oracle.HIER, coarse=NL, fine=F).stats
    n_ckpt = -(-T // F)
    batches = -(-n_ckpt // NL)
    assert st["local_slots"] == F + NL
    assert st["remote_writes"] == batches - 1 and st["remote_reads"] == batches - 1
    assert st["remote_slots"] == (batches - 1) * NL
    assert (st["fwd_steps"], st["refwd1_steps"], st["refwd2_steps"], st["bwd_steps"]) == (T, 0, T, T)


def test_sqrt_rules_minimise_local_memory():
    """chunk = sqrt(T) minimises Chunk's slots (64 for T = 4096, Hyperparameter Study) and
    chunk = sqrt(remote_chunk) minimises Double's; Double's minimum over both grows like T^(1/4)."""
    def chunk_slots(T, F):
        return F + -(-T // F)

    def double_slots(C, F):
        return F + -(-C // F)
    assert min(range(1, 4097), key=lambda F: chunk_slots(4096, F)) == 64
    assert min(range(1, 257), key=lambda F: double_slots(256, F)) == 16
    net = _tiny(9, T=256, B=1, hidden=(3,))
    assert _run(net, strategy=oracle.CHUNK, fine=16, backward=False).stats["local_slots"] == chunk_slots(256, 16)
    assert _run(net, strategy=oracle.DOUBLE, coarse=64, fine=8, backward=False).stats["local_slots"] == double_slots(64, 8)


def test_openmp_batch_parallel_matches_serial():
    w = synth.config(0, B=6)
    d = synth.generate(w)
    args = (w.n_in, list(w.n_hidden), w.n_out, d["W_in"], d["W_rec"], d["W_out"], d["in_spikes"], d["labels"])
    a = oracle.bptt(*args, nthreads=1)
    b = oracle.bptt(*args, nthreads=3)
    assert b.stats["threads_used"] == 3
    assert np.array_equal(a.spikes[0], b.spikes[0]) and abs(a.loss - b.loss) < 1e-12
    for p, q in zip(a.dW_in + a.dW_rec + [a.dW_out], b.dW_in + b.dW_rec + [b.dW_out]):
        assert np.allclose(p, q, rtol=0, atol=1e-5 * np.abs(p).max())


def test_invalid_intervals_rejected():
    net = _tiny(1)
    with pytest.raises(ValueError):
        _run(net, strategy=oracle.DOUBLE, coarse=3, fine=5)
    with pytest.raises(ValueError):
        _run(net, strategy=oracle.CHUNK, fine=0)


def test_forced_states_mode_is_consistent():
    """Feeding the double-precision oracle its own states changes nothing; feeding it the fp32
    trajectory moves the gradients only by the fp32 rounding of the states."""
    net = _tiny(23, n_in=10, hidden=(12, 8), T=20, B=2, p=0.25, scale=0.6)
    a = _run(net, dtype=np.float64, want_v=True)
    b = _run(net, dtype=np.float64, forced_spikes=a.spikes, forced_v=a.v)
    for p, q in zip(a.dW_in + a.dW_rec + [a.dW_out], b.dW_in + b.dW_rec + [b.dW_out]):
        assert np.array_equal(p, q)
    f = _run(net, dtype=np.float32, want_v=True)
    assert all(np.array_equal(x, y) for x, y in zip(f.spikes, a.spikes))
    c = _run(net, dtype=np.float64, forced_spikes=f.spikes, forced_v=f.v)
    for p, q in zip(a.dW_in + a.dW_rec, c.dW_in + c.dW_rec):
        assert np.allclose(p, q, rtol=0, atol=1e-4 * np.abs(p).max()) and not np.array_equal(p, q)
    with pytest.raises(ValueError):
        _run(net, dtype=np.float64, forced_spikes=a.spikes, forced_v=a.v, strategy=oracle.CHUNK, fine=4)


def test_gradient_reference_for_the_gpu_parity_bar():
    """Why the GPU gradients are compared with the oracle's backward pass in fp64 on the fp32 forward trajectory,
    and not with the fp32 oracle's own gradients (configuration 1 at its full size: T = 1000, batch 32).
    The fp32 oracle adds the ~16 000 terms of a dW_out element one after the other in fp32; with one thread and
    with eight (private partial sums per thread, reduced in thread order) it is the same arithmetic in a different
    grouping.  Pinned here: (1) the forward trajectory -- spikes and membrane potentials -- does not depend on the
    grouping, bit for bit; (2) the two fp32 gradient sets differ from each other by more than the 1e-4 parity
    bar on dW_out, and the sequential one is more than 1e-4 away from the fp64 evaluation: an fp32 sequential sum
    cannot referee a 1e-4 bar; (3) the fp64 evaluation on that same trajectory does not depend on the grouping
    (spread < 1e-10), and the better-conditioned of the fp32 sums (eight partial sums) agrees with it to well
    inside the bar, so it sits where the fp32 results scatter around."""
    w = synth.config(1)
    d = synth.generate(w)

    def run(dtype, nthreads, **kw):
        return oracle.bptt(w.n_in, list(w.n_hidden), w.n_out, d["W_in"], d["W_rec"], d["W_out"], d["in_spikes"],
                           d["labels"], dtype=dtype, nthreads=nthreads, **kw)

    def tensors(r):
        return list(r.dW_in) + list(r.dW_rec) + [r.dW_out]

    def rel(a, b, scale):
        return float(np.abs(a - b).max() / np.abs(scale).max())

    f1 = run(np.float32, 1, want_v=True)
    f8 = run(np.float32, 8, want_v=True)
    for l in range(len(w.n_hidden)):
        assert np.array_equal(f1.spikes[l], f8.spikes[l]) and np.array_equal(f1.v[l], f8.v[l])
    forced = dict(forced_spikes=[s.astype(np.float64) for s in f1.spikes], forced_v=[v.astype(np.float64) for v in f1.v])
    r4 = run(np.float64, 4, **forced)
    r8 = run(np.float64, 8, **forced)
    spread32 = [rel(a, b, c) for a, b, c in zip(tensors(f1), tensors(f8), tensors(r8))]
    off_seq = [rel(a, c, c) for a, c in zip(tensors(f1), tensors(r8))]
    off_par = [rel(a, c, c) for a, c in zip(tensors(f8), tensors(r8))]
    spread64 = [rel(a, b, b) for a, b in zip(tensors(r4), tensors(r8))]
    print("fp32 1 vs 8 threads:", spread32, "\nfp32 sequential vs fp64:", off_seq, "\nfp32 8 partials vs fp64:", off_par,
          "\nfp64 4 vs 8 threads:", spread64)
    assert spread32[-1] > 1e-4 and off_seq[-1] > 1e-4          # dW_out: measured 2.0e-4 and 1.9e-4
    assert max(spread64) < 1e-10                                # measured 3e-13
    assert max(off_par) < 5e-5                                  # measured 1.4e-5


def test_loss_gradient_of_a_confident_softmax():
    """d loss / d ubar = softmax - onehot, checked against 60-digit decimal arithmetic where the softmax is
    saturated (the labelled class's probability is 1 - 1e-13 and less): the readout weights are scaled until the
    time-averaged readouts are tens of units apart.  dW_out is linear in that gradient (dW_out[j] = sum over the
    steps where neuron j fired of du_t, du_t = beta du_{t+1} + g), so it is rebuilt in decimal arithmetic from the
    oracle's own spike train and compared.  Formed as a difference of numbers near one the labelled class's entry
    would be off by 1e-3 here; as minus the sum of the other classes' probabilities it keeps full precision."""
    from decimal import Decimal, getcontext
    getcontext().prec = 60
    net = _tiny(5, hidden=(6,), n_out=3, T=9, B=2)
    beta = 0.75  # exact in binary and in decimal
    checked = 0
    W0 = net["W_out"].copy()
    for scale in (40.0, 100.0):
        net["W_out"] = np.round(W0 * scale * 64) / 64  # dyadic: the decimal copy is exact
        first = oracle.bptt(net["n_in"], net["n_hidden"], net["n_out"], net["W_in"], net["W_rec"], net["W_out"],
                            net["in_spikes"], net["labels"], dtype=np.float64, beta=beta, backward=False)
        net["labels"] = first.ubar.argmax(axis=1).astype(np.int32)  # confident and right: softmax_y -> 1
        r = oracle.bptt(net["n_in"], net["n_hidden"], net["n_out"], net["W_in"], net["W_rec"], net["W_out"],
                        net["in_spikes"], net["labels"], dtype=np.float64, beta=beta)
        T, B = net["in_spikes"].shape[:2]
        N, O = net["W_out"].shape
        Wd = [[Decimal(float(net["W_out"][j, o])) for o in range(O)] for j in range(N)]
        exp_dW = [[Decimal(0)] * O for _ in range(N)]
        for b in range(B):
            u = [Decimal(0)] * O
            usum = [Decimal(0)] * O
            for t in range(T):
                cur = [sum((Wd[j][o] for j in range(N) if r.spikes[0][t, b, j] != 0), Decimal(0)) for o in range(O)]
                u = [Decimal(beta) * u[o] + cur[o] for o in range(O)]
                usum = [usum[o] + u[o] for o in range(O)]
            ubar = [x / T for x in usum]
            m = max(ubar)
            e = [(x - m).exp() for x in ubar]
            z = sum(e)
            y = int(net["labels"][b])
            g = [(e[o] / z - (1 if o == y else 0)) / (B * T) for o in range(O)]
            one_minus_py = 1 - e[y] / z
            if Decimal(0) < one_minus_py < Decimal("1e-12"):
                checked += 1
            du = [Decimal(0)] * O
            for t in reversed(range(T)):
                du = [Decimal(beta) * du[o] + g[o] for o in range(O)]
                for j in range(N):
                    if r.spikes[0][t, b, j] != 0:
                        exp_dW[j] = [exp_dW[j][o] + du[o] for o in range(O)]
        exp = np.array([[float(x) for x in row] for row in exp_dW])
        assert np.abs(exp).max() > 0
        err = np.abs(r.dW_out - exp).max() / np.abs(exp).max()
        assert err < 1e-11, (scale, err)
    assert checked >= 1  # at least one batch element was saturated beyond fp64's rounding step of 1
