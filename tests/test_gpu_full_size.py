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
