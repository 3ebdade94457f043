"""snn_forward_noalloc (the entry point for callers that cannot allocate device memory) against snn_forward:
same spike trains, readout and loss bit for bit, on two calls in a row, the second with a shorter sequence;
sizes beyond its static workspace and host pointers are refused with an error, nothing runs."""
import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu

snn = pytest.importorskip("paper_2412_11810_amd")


def _forward_result(net, L, T):
    ubar, loss = net.snn_get_readout()
    return [net.snn_get_spikes(l, T) for l in range(L)], ubar, loss


def test_forward_without_allocation_matches_snn_forward():
    torch = pytest.importorskip("torch")
    w = synth.config(1, T=150, B=6)
    d = synth.generate(w)
    L = len(w.n_hidden)
    x = torch.from_numpy(d["in_spikes"]).cuda()
    y = torch.from_numpy(d["labels"]).cuda()
    ref_net = snn.from_workload(w, d)
    net = snn.from_workload(w, d)
    try:
        for T in (150, 40):  # the second call is smaller: what the first left in the workspace must not matter
            xs = x[:T].contiguous()
            loss_ref = ref_net.snn_forward(xs, y, T)
            spikes_ref, ubar_ref, _ = _forward_result(ref_net, L, T)
            loss = net.snn_forward_noalloc(xs, y, T)
            spikes, ubar, loss2 = _forward_result(net, L, T)
            assert np.float32(loss) == np.float32(loss_ref) == np.float32(loss2)
            assert np.array_equal(ubar.view(np.uint32), ubar_ref.view(np.uint32))
            for a, b in zip(spikes, spikes_ref):
                assert np.array_equal(a, b) and a.sum() > 0
        # the inputs are bound: a training step follows without another forward call, and matches
        net.snn_bptt(snn.SNN_CHUNK, 0, 16)
        ref_net.snn_bptt(snn.SNN_CHUNK, 0, 16)
        for kind, layer in ((snn.SNN_W_IN, 0), (snn.SNN_W_REC, 1), (snn.SNN_W_OUT, 0)):
            assert np.array_equal(net.snn_grads(kind, layer), ref_net.snn_grads(kind, layer))
        with pytest.raises(snn.SnnError) as e:
            net.snn_forward_noalloc(d["in_spikes"][:40].copy(), d["labels"], 40)  # host pointers
        assert e.value.status == snn.SNN_E_INVAL
        bad = y.clone()
        bad[0] = w.n_out
        with pytest.raises(snn.SnnError) as e:
            net.snn_forward_noalloc(x[:40].contiguous(), bad, 40)
        assert e.value.status == snn.SNN_E_INVAL and "label" in str(e.value)
    finally:
        net.snn_destroy()
        ref_net.snn_destroy()


def test_forward_without_allocation_refuses_networks_beyond_its_workspace():
    torch = pytest.importorskip("torch")
    w = synth.config(2, T=8)  # 64 * 64 * (160 + 2 * 3072) * 4 B = 103 MB of per-tile currents
    d = synth.generate(w)
    net = snn.from_workload(w, d)
    try:
        x = torch.from_numpy(d["in_spikes"]).cuda()
        y = torch.from_numpy(d["labels"]).cuda()
        with pytest.raises(snn.SnnError) as e:
            net.snn_forward_noalloc(x, y, w.T)
        assert e.value.status == snn.SNN_E_INVAL and "16777216" in str(e.value)
        assert net.snn_forward(x, y, w.T) > 0.0  # the allocating entry point still serves it
    finally:
        net.snn_destroy()
