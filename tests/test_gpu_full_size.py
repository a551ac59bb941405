"""HIP path vs CPU oracle on the network of the headline benchmark at its full size
(100,000 neurons x fan-out 1,000 = 1e8 synapses, delays 1..250 steps), in the launch
configuration bench.py times (same grids, same window length, same staging regions).

The oracle needs minutes for the benchmark's 1,000 steps, so the run here is 300 steps (longer
than the largest delay, so the circular spike history wraps) with a drive of 55 Hz, which
makes the network emit 2.5e7 events in them; everything is compared: the membrane trace bit
for bit, all counters, and every entry of both gradients.

The batched configuration (256 trials of 4,096 neurons: 2^20 state cells, the largest grids of
the step kernels) is run the same way at its full batch for 200 steps.
"""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2512_05906_amd import adseq, synth
from tests import helpers as H

pytestmark = pytest.mark.gpu

T = 300


@pytest.fixture(scope="module")
def wl():
    return synth.cfg3(rate_hz=55.0, n_steps=T)


@pytest.mark.parametrize("kind,cap", [("ring", 0), ("fifo", 32), ("latest", 1)])
def test_cfg3_full_size_forward_backward(wl, kind, cap):
    k = {"ring": oracle.RING, "fifo": oracle.FIFO, "latest": oracle.SYN_LATEST}[kind]
    print(f"cfg3 full size, {kind}[{cap}], T={T}: oracle forward", flush=True)
    ref = oracle.Run(wl, k, cap, n_steps=T)
    rc = ref.counters()
    counts = ref.spikes.sum(axis=0).astype(np.float32)
    y = synth.spike_count_targets(wl)
    dL_dc = (2.0 * (counts - y) / np.float32(wl.n_neurons)).astype(np.float32)
    print("oracle backward", flush=True)
    gw, gd = ref.backward(dL_dc, None)
    U_ref = ref.U
    ref.close()

    print("GPU forward + backward", flush=True)
    spike_cap = 4 * wl.n_neurons
    sim = adseq.Adseq(wl, k, cap, record_tape=True, max_steps=T, tape_spike_capacity=spike_cap,
                      tape_event_capacity=(spike_cap * wl.fan_out if kind != "ring" else 0))
    sim.run(0, T)
    torch.cuda.synchronize()
    U = sim.tape()["U"].cpu().numpy()
    np.testing.assert_array_equal(U.view(np.uint32), U_ref.view(np.uint32))
    c = sim.counters()
    for key in ("enqueued", "dropped", "delivered", "sum_enqueued", "sum_dropped", "sum_delivered"):
        assert c[key] == rc[key], key
    assert c["error_bits"] == 0
    assert rc["enqueued"] > 2e7 and rc["delivered"] > 4e6
    if kind == "fifo":
        assert rc["dropped"] > 1e7
    if kind == "latest":     # one slot per synapse and trial: 1e8 queues, looked at in every step
        assert rc["dropped"] > 1e5
    cnt = torch.empty(wl.n_neurons, dtype=torch.int32, device=sim.dev)
    sim.spike_counts(cnt)
    np.testing.assert_array_equal(cnt.cpu().numpy(), counts.astype(np.int32).reshape(-1))
    g_w = torch.full((wl.n_synapses,), 7.0, dtype=torch.float32, device=sim.dev)
    g_d = torch.full((wl.n_synapses,), 7.0, dtype=torch.float32, device=sim.dev)
    sim.backward(torch.from_numpy(dL_dc).to(sim.dev), None, g_w, g_d)
    torch.cuda.synchronize()
    H.grad_close(g_w.cpu().numpy(), gw)
    H.grad_close(g_d.cpu().numpy(), gd)
    assert np.abs(gw).max() > 0 and np.abs(gd).max() > 0
    sim.close()


@pytest.mark.parametrize("kind,cap,drive_hz", [("ring", 0, 10.0), ("ring", 0, 100.0), ("fifo", 32, 250.0), ("sorted", 128, 10.0)])
def test_cfg4_full_batch_forward_backward(kind, cap, drive_hz):
    """Config 4 with all 256 trials (2^20 state cells, 4,096 blocks per step launch, 4,096 target
    parts in the ring's window expansion, continuous delays), 200 steps: with the drive the
    config prescribes (a few spikes per step: the sparse route of the window expansion) and with
    a strong one (the staged route at this size; bounded queues that hold many events)."""
    Tc = 200
    w = synth.cfg4(n_steps=Tc)
    w.ext_rate_hz = drive_hz
    k = {"ring": oracle.RING, "fifo": oracle.FIFO, "sorted": oracle.SORTED}[kind]
    print(f"cfg4 full batch, {kind}[{cap}], drive {drive_hz} Hz, T={Tc}: oracle", flush=True)
    ref = oracle.Run(w, k, cap, n_steps=Tc, n_threads=16)
    rc = ref.counters()
    counts = ref.spikes.sum(axis=0).astype(np.float32)
    y = synth.spike_count_targets(w)
    dL_dc = (2.0 * (counts - y) / np.float32(w.batch * w.n_neurons)).astype(np.float32)
    gw, gd = ref.backward(dL_dc, None)
    U_ref = ref.U
    ref.close()
    print("GPU forward + backward", flush=True)
    spike_cap = max(1 << 16, 2 * int(counts.sum()))
    sim = adseq.Adseq(w, k, cap, record_tape=True, max_steps=Tc, tape_spike_capacity=spike_cap,
                      tape_event_capacity=(spike_cap * w.fan_out if kind != "ring" else 0))
    sim.run(0, Tc)
    torch.cuda.synchronize()
    U = sim.tape()["U"].cpu().numpy()
    np.testing.assert_array_equal(U.view(np.uint32), U_ref.view(np.uint32))
    c = sim.counters()
    for key in ("enqueued", "dropped", "delivered", "sum_enqueued", "sum_dropped", "sum_delivered"):
        assert c[key] == rc[key], key
    assert c["error_bits"] == 0
    assert rc["enqueued"] > (1e7 if drive_hz >= 100 else 1e5)
    g_w = torch.full((w.n_synapses,), 7.0, dtype=torch.float32, device=sim.dev)
    g_d = torch.full((w.n_synapses,), 7.0, dtype=torch.float32, device=sim.dev)
    sim.backward(torch.from_numpy(dL_dc.reshape(-1)).to(sim.dev), None, g_w, g_d)
    torch.cuda.synchronize()
    H.grad_close(g_w.cpu().numpy(), gw)
    H.grad_close(g_d.cpu().numpy(), gd)
    assert np.abs(gw).max() > 0 and np.abs(gd).max() > 0
    sim.close()


@pytest.mark.parametrize("kind,cap", [("ring", 0), ("fifo", 32)])
def test_cfg3_bench_run_properties(kind, cap):
    """The run bench.py times (1,000 steps, the drive tuned for 20 Hz), where the oracle would need
    minutes: what must hold at any size.  Two runs give the same bits in the membrane trace and the
    counters (integer sums: nothing depends on the order in which atomics land) and the same
    gradients up to the order of a synapse's fp32 terms; the events that are
    neither delivered nor dropped number no more than the queues can still hold; the spike counts
    and the offered events are those of the recorded trace."""
    w = synth.cfg3()
    k = {"ring": adseq.RING, "fifo": adseq.FIFO}[kind]
    Tb = w.n_steps
    spike_cap = 4 * w.n_neurons
    sim = adseq.Adseq(w, k, cap, record_tape=True, max_steps=Tb, tape_spike_capacity=spike_cap,
                      tape_event_capacity=(spike_cap * w.fan_out if kind != "ring" else 0))
    y = torch.from_numpy(synth.spike_count_targets(w).reshape(-1)).to(sim.dev)
    runs = []
    for rep in range(2):
        print(f"cfg3 bench run, {kind}[{cap}], pass {rep}", flush=True)
        if rep:
            sim.reset()
        sim.run(0, Tb)
        cnt = torch.empty(w.n_neurons, dtype=torch.int32, device=sim.dev)
        sim.spike_counts(cnt)
        dL_dc = 2.0 * (cnt.float() - y) / w.n_neurons
        g_w = torch.full((w.n_synapses,), 7.0, dtype=torch.float32, device=sim.dev)
        g_d = torch.full((w.n_synapses,), 7.0, dtype=torch.float32, device=sim.dev)
        sim.backward(dL_dc, None, g_w, g_d)
        torch.cuda.synchronize()
        U = sim.tape()["U"]
        c = sim.counters()
        assert c["error_bits"] == 0
        in_flight = c["enqueued"] - c["delivered"] - c["dropped"]
        # what is neither delivered nor dropped is still stored: at most what the queues hold
        # (bounded kinds), at most the events of the last d_max steps' spikes (ring)
        last = int((U[Tb - w.d_max_steps:] >= w.v_thresh).sum().item()) * w.fan_out
        assert 0 <= in_flight <= (min(cap * w.n_neurons, last) if kind != "ring" else last)
        spikes = int((U >= w.v_thresh).sum().item())
        assert int(cnt.sum().item()) == spikes and c["enqueued"] == spikes * w.fan_out
        assert bool(torch.isfinite(g_w).all()) and bool(torch.isfinite(g_d).all())
        assert float(g_w.abs().max()) > 0 and float(g_d.abs().max()) > 0
        runs.append((U.clone(), g_w, g_d, c))
    assert torch.equal(runs[0][0].view(torch.int32), runs[1][0].view(torch.int32))
    # gradients: the same up to the order in which the terms of one synapse are added (two spikes
    # of one neuron whose events land in the same window are gathered by the same launch)
    for a, b in ((runs[0][1], runs[1][1]), (runs[0][2], runs[1][2])):
        assert float((a - b).norm()) <= 1e-6 * float(a.norm())
        assert float((a - b).abs().max()) <= 1e-5 * float(a.abs().max())
    assert runs[0][3] == runs[1][3]
    if kind == "ring":
        assert runs[0][3]["dropped"] == 0 and 15.0 < spikes / (w.n_neurons * Tb * w.dt_ms * 1e-3) < 25.0
    else:
        assert runs[0][3]["dropped"] > 1e7
    sim.close()
