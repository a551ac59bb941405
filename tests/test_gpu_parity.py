"""HIP path vs CPU oracle, element by element, through the C ABI (needs an MI355X)."""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2512_05906_amd import adseq, synth
from tests import helpers as H

pytestmark = pytest.mark.gpu

KINDS = {"ring": oracle.RING, "fifo": oracle.FIFO, "sorted": oracle.SORTED, "syn": oracle.SYN_FIFO, "latest": oracle.SYN_LATEST, "bins": oracle.SYN_BINS}


def _compare_forward(wl, kind, cap, T=None, B=None, i_ext=None, check_sets=True, **kw):
    T = wl.n_steps if T is None else T
    B = wl.batch if B is None else B
    ref = oracle.Run(wl, kind, cap, n_steps=T, batch=B, i_ext=i_ext, log_events=True, n_threads=8)
    sim, out = H.run_gpu(wl, kind, cap, n_steps=T, batch=B, i_ext=i_ext, **kw)
    np.testing.assert_array_equal(out["S"], ref.spikes)                 # raster, bit exact
    np.testing.assert_array_equal(out["U"].view(np.uint32), ref.U.view(np.uint32))  # membrane, bit exact
    if kind != oracle.RING:
        np.testing.assert_array_equal(H.spikes_from_tape(out, wl, B), ref.spikes)
    else:
        np.testing.assert_array_equal(out["U"] >= np.float32(wl.v_thresh), ref.spikes.astype(bool))
    c, rc = out["counters"], ref.counters()
    for key in ("enqueued", "dropped", "delivered", "sum_enqueued", "sum_dropped", "sum_delivered"):
        assert c[key] == rc[key], key
    assert c["error_bits"] == 0
    assert sim.drop_count() == dict(dropped=rc["dropped"], enqueued=rc["enqueued"], delivered=rc["delivered"])
    if kind != oracle.RING and check_sets:
        adm, drp = H.gpu_dropped_set(sim, out, wl)
        o_del, o_drp = H.oracle_sets(ref)
        assert drp == o_drp                                              # dropped-event set
        in_run = {(p, n, b) for (p, n, b) in adm if n + int(ref.D[p]) < T}
        assert in_run == o_del                                           # delivered-event set
    sim.close()
    return ref, out


@pytest.mark.parametrize("kind", ["ring", "sorted", "fifo", "syn"])
def test_cfg0_forward_lossless(kind):
    """Config 0 with the ring and with the exact ordered queue (capacity = the
    largest occupancy the oracle sees, so nothing is dropped)."""
    wl = synth.cfg0()
    cap = oracle.Run(wl, KINDS[kind], 10**6).counters()["max_occupancy"] if kind != "ring" else 0
    ref, out = _compare_forward(wl, KINDS[kind], cap)
    assert ref.counters()["dropped"] == 0 and ref.spikes.sum() > 100


@pytest.mark.parametrize("kind,cap", [("fifo", 1), ("fifo", 3), ("sorted", 2), ("sorted", 5)])
def test_cfg0_forward_lossy(kind, cap):
    wl = synth.cfg0(seed=11)
    wl.ext_rate_hz = 120.0
    ref, _ = _compare_forward(wl, KINDS[kind], cap)
    assert ref.counters()["dropped"] > 0


@pytest.mark.parametrize("kind,cap", [("ring", 0), ("fifo", 4), ("sorted", 4), ("syn", 1), ("latest", 1), ("bins", 3)])
@pytest.mark.parametrize("continuous", [False, True])
def test_ragged_rows_batched(kind, cap, continuous):
    """Rows of 0..700 synapses (several 256-wide tiles plus a ragged tail, empty rows,
    duplicate targets), 3 trials, heavy drive so that the bounded kinds overflow."""
    wl = synth.ragged_network(300, 700, 37, seed=5, rate_hz=300.0, t=120, b=3, continuous=continuous,
                              w_mean=0.004, w_std=0.003)
    ref, _ = _compare_forward(wl, KINDS[kind], cap, check_sets=(kind != "ring"))
    assert ref.spikes.sum() > 300
    if kind != "ring":
        assert ref.counters()["dropped"] > (1000 if kind not in ("syn", "latest", "bins") else 100)


@pytest.mark.parametrize("cap", [1, 2, 3, 8])
def test_per_synapse_queues_bursty(cap):
    """One bounded FIFO per synapse (Section 4.1 listing 1, Section 4.3 "FIFORing"): neurons that
    fire in bursts, so that a synapse often holds several events; rasters, membrane values,
    counters and the dropped / delivered event sets against the oracle."""
    wl = synth.ragged_network(200, 90, 25, seed=6, rate_hz=3000.0, t=200, b=3, w_mean=0.02, w_std=0.02)
    ref, _ = _compare_forward(wl, oracle.SYN_FIFO, cap, tape_spike_capacity=200 * 3 * 200)
    assert ref.spikes.sum() > 2000
    if cap < 8:
        assert ref.counters()["dropped"] > 500


@pytest.mark.parametrize("bins", [1, 2, 3, 8])
def test_time_bins_bursty(bins):
    """Time bins per synapse (Section 4.3 "LossyRingDelay(n)": bin = arrival step mod n, the newer
    event takes the bin): bursting neurons; rasters, membrane values, counters and the lost /
    delivered event sets (from the admission flags) against the oracle."""
    wl = synth.ragged_network(200, 90, 25, seed=6, rate_hz=3000.0, t=200, b=3, w_mean=0.02, w_std=0.02)
    ref, _ = _compare_forward(wl, oracle.SYN_BINS, bins, tape_spike_capacity=200 * 3 * 200)
    assert ref.spikes.sum() > 2000 and ref.counters()["dropped"] > 500


def test_latest_spike_slots_bursty():
    """One slot per synapse that always takes the newest spike (Section 4.3 "SingleSpike(Drop)"):
    bursting neurons, so that many held events are replaced before they arrive; rasters, membrane
    values, counters and the lost / delivered event sets (from the admission flags, which the push
    that replaces an event clears) against the oracle."""
    wl = synth.ragged_network(200, 90, 25, seed=6, rate_hz=3000.0, t=200, b=3, w_mean=0.02, w_std=0.02)
    ref, _ = _compare_forward(wl, oracle.SYN_LATEST, 1, tape_spike_capacity=200 * 3 * 200)
    assert ref.spikes.sum() > 2000 and ref.counters()["dropped"] > 500


@pytest.mark.parametrize("window", [2, 8, 16, 64])
@pytest.mark.parametrize("stage", [0, 1, 700])
def test_ring_window_length_and_staging_capacity(window, stage, monkeypatch):
    """The ring's results depend neither on the window length nor on the capacity of the
    staging buffer of the window expansion: default (everything staged), 1 event (every far
    event takes the atomic fallback), 700 events (regions overflow: both routes mixed)."""
    monkeypatch.setenv("ADSEQ_RING_WINDOW", str(window))
    wl = synth.ragged_network(300, 700, 37, seed=5, rate_hz=300.0, t=150, b=3,
                              w_mean=0.004, w_std=0.003)
    ref, _ = _compare_forward(wl, oracle.RING, 0, step_event_capacity=stage)
    assert ref.spikes.sum() > 300


def test_ring_row_data_fetched_by_spiking_lanes_only(monkeypatch):
    """ADSEQ_RING_LAZY_ROWS = 1: the step kernels load row start, in-window count and far queue
    term for spiking lanes only (less traffic, one more round trip): same trace, counters, event
    sets and gradients."""
    monkeypatch.setenv("ADSEQ_RING_LAZY_ROWS", "1")
    wl = synth.ragged_network(900, 300, 37, seed=15, rate_hz=300.0, t=150, b=3, w_mean=0.004, w_std=0.003)
    ref, _ = _compare_forward(wl, oracle.RING, 0)
    assert ref.spikes.sum() > 300
    _compare_backward(wl, oracle.RING, 0, 150, 3)


@pytest.mark.parametrize("rate_hz", [40.0, 80.0, 160.0])
def test_ring_sparse_windows_take_atomics_block_by_block(rate_hz):
    """48,000 state cells (188 target parts) and a firing rate that climbs from zero: a block of
    the window expansion with fewer events than parts adds them to the window directly and leaves
    its staging counters untouched, one with more stages them, so a run passes through windows
    of either sort and windows in which the blocks differ (the results do not: integer sums)."""
    wl = synth.ragged_network(3000, 40, 60, seed=33, rate_hz=rate_hz, t=200, b=16, w_mean=0.01, w_std=0.01)
    ref, _ = _compare_forward(wl, oracle.RING, 0, check_sets=False)
    assert ref.spikes.sum() > 1000


def test_ring_rows_longer_than_a_staging_chunk():
    """Rows of up to 60,000 synapses with delays of 1..6 steps: the piece of a row that lands in
    one window (4 steps here) holds tens of thousands of events, so one piece spans several of
    the 8,192-event chunks in which the window expansion orders its events, and 40 targets make
    a single target part."""
    wl = synth.ragged_network(40, 60000, 6, seed=21, rate_hz=300.0, t=80, b=1, w_mean=0.00002, w_std=0.00002,
                              empty_rows=False)
    ref, _ = _compare_forward(wl, oracle.RING, 0)
    assert ref.spikes.sum() > 20 and ref.counters()["enqueued"] > 500000


@pytest.mark.parametrize("kind,cap", [("ring", 0), ("fifo", 5), ("sorted", 5), ("syn", 2), ("latest", 1), ("bins", 5)])
def test_largest_delay_range(kind, cap):
    """Delays up to the largest the interface allows (1,023 steps) over a run longer than that, so
    that the delay line, the spike history and the arrival keys wrap around; forward and both
    gradients."""
    wl = synth.ragged_network(90, 60, 1023, seed=33, rate_hz=120.0, t=1500, b=2, w_mean=0.03, w_std=0.03)
    # delays spread over the whole range, with both ends present
    rng = np.random.default_rng(33)
    d = rng.integers(1, 1024, size=wl.n_synapses)
    d[:4] = (1, 1023, 1022, 2)
    wl.delay_steps = None
    wl.delay_ms = (d.astype(np.float32) * np.float32(wl.dt_ms)) - np.float32(0.03)   # continuous, just short of the grid
    # (a small membrane cotangent: over 1,500 steps the gradient entries are sums of thousands of
    # terms that partly cancel, and fp32 keeps 1e-6 absolute only if the terms are not large)
    ref = _compare_backward(wl, KINDS[kind], cap, 1500, 2, dU_scale=1e-4, tape_spike_capacity=1500 * 2 * 90)
    assert ref.spikes.sum() > 300 and int(ref.D.max()) == 1023 and int(ref.D.min()) == 1


@pytest.mark.parametrize("kind,cap", [("ring", 0), ("fifo", 2), ("sorted", 2), ("syn", 1), ("latest", 1), ("bins", 2)])
def test_degenerate_networks(kind, cap):
    """One neuron that talks to itself through three synapses (every block, word and part has a
    single valid lane), and a network without any synapse (empty rows only, nothing ever queued)."""
    one = synth.Workload(name="one", n_neurons=1, fan_out=3, n_steps=300, batch=3, d_max_steps=4,
                         ext_rate_hz=900.0, seed=8, row_ptr=np.array([0, 3], np.int64),
                         col=np.zeros(3, np.int32), weight=np.array([0.3, -0.1, 0.25], np.float32),
                         delay_steps=np.array([1, 4, 2], np.uint8))
    ref = _compare_backward(one, KINDS[kind], cap, 300, 3, tape_spike_capacity=900)
    assert ref.spikes.sum() > 30
    if kind != "ring":
        assert ref.counters()["dropped"] > 0
    none = synth.Workload(name="none", n_neurons=70, fan_out=0, n_steps=100, batch=2, d_max_steps=5,
                          ext_rate_hz=900.0, seed=9, row_ptr=np.zeros(71, np.int64),
                          col=np.zeros(0, np.int32), weight=np.zeros(0, np.float32),
                          delay_steps=np.zeros(0, np.uint8))
    ref, out = _compare_forward(none, KINDS[kind], cap, check_sets=False)
    assert ref.spikes.sum() > 100 and out["counters"]["enqueued"] == 0


@pytest.mark.parametrize("window", [4, 32])
def test_ring_backward_other_window_lengths(window, monkeypatch):
    monkeypatch.setenv("ADSEQ_RING_WINDOW", str(window))
    wl = synth.ragged_network(120, 300, 30, seed=12, rate_hz=300.0, t=150, b=2, continuous=True,
                              w_mean=0.01, w_std=0.01)
    _compare_backward(wl, oracle.RING, 0, 150, 2)


def test_external_current_and_no_drive():
    wl = synth.cfg0(seed=3)
    wl.ext_rate_hz = 0.0
    rng = np.random.default_rng(0)
    i_ext = (rng.random((200, 2, 100)) * 0.02).astype(np.float32)
    ref, _ = _compare_forward(wl, oracle.RING, 0, T=200, B=2, i_ext=i_ext)
    assert ref.spikes.sum() > 10


def test_no_spikes_and_zero_steps():
    wl = synth.cfg0(seed=3)
    wl.ext_rate_hz = 0.0
    ref, out = _compare_forward(wl, oracle.FIFO, 2, T=50)
    assert ref.spikes.sum() == 0 and out["counters"]["enqueued"] == 0
    sim, out = H.run_gpu(wl, oracle.RING, 0, n_steps=0, record=False)
    assert out["counters"]["delivered"] == 0


@pytest.mark.parametrize("kind,cap", [("ring", 0), ("fifo", 2), ("sorted", 3), ("syn", 1), ("latest", 1), ("bins", 2)])
def test_open_loop_enqueue_deliver(kind, cap):
    """adseq_enqueue / adseq_deliver with externally generated spike lists (the
    shape of the paper's Poisson benchmark, Section 5.1)."""
    wl = synth.ragged_network(200, 40, 25, seed=9, rate_hz=0.0, t=150, b=2)
    T, B, N = 150, 2, 200
    lists = synth.poisson_spike_lists(N, B, T, 400.0, wl.dt_ms, seed=4)
    forced = np.zeros((T, B * N), np.uint8)
    for n, ids in enumerate(lists):
        forced[n, ids] = 1
    forced = forced.reshape(T, B, N)
    ref = oracle.Run(wl, KINDS[kind], cap, n_steps=T, batch=B, forced_spikes=forced, keep_currents=True)
    sim = adseq.Adseq(wl, KINDS[kind], cap, batch=B)
    I = torch.zeros((T, B, N), dtype=torch.float32, device=sim.dev)
    for n in range(T):
        sim.deliver(n, I[n])
        ids = torch.from_numpy(lists[n]).to(sim.dev)
        cnt = torch.tensor([len(lists[n])], dtype=torch.int32, device=sim.dev)
        sim.enqueue(n, ids, cnt)
    torch.cuda.synchronize()
    want = ref.Iq.astype(np.float32) * np.float32(2.0 ** -24)
    np.testing.assert_array_equal(I.cpu().numpy().view(np.uint32), want.view(np.uint32))
    c, rc = sim.counters(), ref.counters()
    for key in ("enqueued", "dropped", "delivered", "sum_delivered"):
        assert c[key] == rc[key], key
    if kind != "ring":
        assert rc["dropped"] > 0
    # out-of-order calls are refused and leave the handle usable
    with pytest.raises(adseq.AdseqError) as ei:
        sim.deliver(T + 5, I[0])
    assert ei.value.code == -4
    sim.deliver(T, I[0])
    sim.close()


def test_run_twice_is_bit_identical_and_reset_works():
    wl = synth.ragged_network(300, 200, 30, seed=6, rate_hz=200.0, t=100, b=2, w_mean=0.01, w_std=0.01)
    sim, a = H.run_gpu(wl, oracle.FIFO, 3, per_step=False)
    sim.reset()
    sim.run(0, 100)
    torch.cuda.synchronize()
    b = sim.tape()["U"].cpu().numpy()
    np.testing.assert_array_equal(a["U"].view(np.uint32), b.view(np.uint32))
    assert sim.counters() == a["counters"]
    sim.close()


def test_ring_repeated_runs_and_mixed_stepping():
    """Several forward + backward passes on one handle, with reset between them and, in one of
    them, single steps followed by adseq_run from the middle of a window: every pass must
    reproduce the oracle (window buffers, staging regions and the slice bookkeeping start clean)."""
    wl = synth.ragged_network(400, 500, 60, seed=21, rate_hz=250.0, t=200, b=2, w_mean=0.006, w_std=0.004)
    T, B = 200, 2
    ref = oracle.Run(wl, oracle.RING, 0, n_steps=T, batch=B, n_threads=8)
    dL_dc = np.full((B, wl.n_neurons), 2e-3, np.float32)
    gw, gd = ref.backward(dL_dc, None)
    sim = adseq.Adseq(wl, adseq.RING, 0, batch=B, record_tape=True, max_steps=T)
    dev = sim.dev
    dc = torch.from_numpy(dL_dc).to(dev)
    g_w = torch.empty(wl.n_synapses, device=dev)
    g_d = torch.empty(wl.n_synapses, device=dev)
    for rep in range(4):
        sim.reset()
        if rep == 2:                       # eager steps first, then the rest as one run
            for n in range(37):
                sim.step(n)
            sim.run(37, T - 37)
        else:
            sim.run(0, T)
        torch.cuda.synchronize()
        U = sim.tape()["U"].cpu().numpy()
        np.testing.assert_array_equal(U.view(np.uint32), ref.U.view(np.uint32))
        c, rc = sim.counters(), ref.counters()
        for key in ("enqueued", "delivered", "sum_enqueued", "sum_delivered"):
            assert c[key] == rc[key], (rep, key)
        g_w.fill_(3.0); g_d.fill_(3.0)
        sim.backward(dc, None, g_w, g_d)
        torch.cuda.synchronize()
        H.grad_close(g_w.cpu().numpy(), gw)
        H.grad_close(g_d.cpu().numpy(), gd)
    sim.close()


def test_create_rejects_bad_delays_and_graph():
    wl = synth.cfg0()
    wl.delay_steps[7] = 0
    with pytest.raises(adseq.AdseqError) as ei:
        adseq.Adseq(wl, adseq.RING)
    assert ei.value.code == -2
    wl = synth.cfg0()
    wl.delay_steps[7] = 21
    with pytest.raises(adseq.AdseqError) as ei:
        adseq.Adseq(wl, adseq.RING)
    assert ei.value.code == -2
    wl = synth.cfg0()
    wl.col[5] = 100
    with pytest.raises(adseq.AdseqError) as ei:
        adseq.Adseq(wl, adseq.RING)
    assert ei.value.code == -8
    wl = synth.cfg0()
    wl.row_ptr[10] = wl.row_ptr[11] + 1
    with pytest.raises(adseq.AdseqError) as ei:
        adseq.Adseq(wl, adseq.RING)
    assert ei.value.code == -8


# ---------------------------------------------------------------- backward

def _compare_backward(wl, kind, cap, T, B, use_dU=True, surrogate=0, dU_scale=1e-3, **kw):
    ref = oracle.Run(wl, kind, cap, n_steps=T, batch=B, surrogate=surrogate, n_threads=8)
    wl_t = synth.Workload(**{**wl.__dict__, "n_steps": T, "batch": B})
    y = synth.spike_count_targets(wl_t)
    counts = ref.spikes.sum(axis=0).astype(np.float32)
    dL_dc = (2.0 * (counts - y) / np.float32(B * wl.n_neurons)).astype(np.float32)
    dL_dU = synth.random_cotangent(wl_t, scale=dU_scale) if use_dU else None
    gw, gd = ref.backward(dL_dc, dL_dU)
    sim, out = H.run_gpu(wl, kind, cap, n_steps=T, batch=B, per_step=False, surrogate=surrogate, **kw)
    np.testing.assert_array_equal(out["U"].view(np.uint32), ref.U.view(np.uint32))
    dev = sim.dev
    g_w = torch.full((wl.n_synapses,), 7.0, dtype=torch.float32, device=dev)  # must be overwritten
    g_d = torch.full((wl.n_synapses,), 7.0, dtype=torch.float32, device=dev)
    sim.backward(torch.from_numpy(dL_dc).to(dev),
                 None if dL_dU is None else torch.from_numpy(dL_dU).to(dev), g_w, g_d)
    torch.cuda.synchronize()
    H.grad_close(g_w.cpu().numpy(), gw)
    H.grad_close(g_d.cpu().numpy(), gd)
    assert np.abs(gw).max() > 0 and np.abs(gd).max() > 0
    sim.close()
    return ref


@pytest.mark.parametrize("kind,cap", [("ring", 0), ("fifo", 4), ("sorted", 6), ("syn", 1), ("latest", 1), ("bins", 2)])
@pytest.mark.parametrize("continuous", [False, True])
def test_backward_small_ragged(kind, cap, continuous):
    wl = synth.ragged_network(120, 300, 30, seed=12, rate_hz=300.0, t=150, b=1, continuous=continuous,
                              w_mean=0.01, w_std=0.01)
    ref = _compare_backward(wl, KINDS[kind], cap, 150, 1, tape_spike_capacity=150 * 120)
    assert ref.spikes.sum() > 100
    if kind != "ring":
        assert ref.counters()["dropped"] > 0


@pytest.mark.parametrize("kind,cap", [("ring", 0), ("fifo", 4), ("sorted", 6), ("syn", 1), ("latest", 1), ("bins", 2)])
@pytest.mark.parametrize("continuous", [False, True])
def test_backward_spike_time_mode(kind, cap, continuous):
    """No surrogate: gradients flow through the emission times of the spikes
    (dt_spk/dv = -1 / vdot, Section 3.1 eq. 8) and the receive rule (eq. 17)."""
    wl = synth.ragged_network(120, 300, 30, seed=14, rate_hz=300.0, t=150, b=2, continuous=continuous,
                              w_mean=0.01, w_std=0.01)
    ref = _compare_backward(wl, KINDS[kind], cap, 150, 2, surrogate=adseq.GRAD_SPIKE_TIME,
                            tape_spike_capacity=2 * 150 * 120)
    assert ref.spikes.sum() > 100
    # the spike-time paths carry weight: the result differs from the one without them
    off = oracle.Run(wl, KINDS[kind], cap, n_steps=150, batch=2, surrogate=oracle.SURR_OFF)
    wl_t = synth.Workload(**{**wl.__dict__, "n_steps": 150, "batch": 2})
    dU = synth.random_cotangent(wl_t, scale=1e-3)
    g_off, _ = off.backward(None, dU)
    g_on, _ = ref.backward(None, dU)
    assert np.linalg.norm(g_on - g_off) > 1e-3 * np.linalg.norm(g_on)


@pytest.mark.parametrize("kind,cap", [("ring", 0), ("fifo", 4), ("sorted", 6)])
@pytest.mark.parametrize("mode", [0, 2])
def test_first_order_synapse_forward_backward(kind, cap, mode):
    """Synaptic current state with its own time constant (Section 2.1 eq. 1): the events jump
    into it, the membrane integrates it; continuous delays decay with that time constant."""
    wl = synth.ragged_network(150, 300, 30, seed=15, rate_hz=250.0, t=160, b=2, continuous=True,
                              w_mean=0.004, w_std=0.004)
    wl.tau_syn_ms = 1.7
    ref = _compare_backward(wl, KINDS[kind], cap, 160, 2, surrogate=mode, tape_spike_capacity=2 * 160 * 150)
    assert ref.spikes.sum() > 100
    plain = oracle.Run(synth.Workload(**{**wl.__dict__, "tau_syn_ms": 0.0}), KINDS[kind], cap, n_steps=160, batch=2)
    assert not np.array_equal(plain.U, ref.U)      # the synaptic state changes the dynamics


@pytest.mark.parametrize("kind,cap", [("ring", 0), ("fifo", 4), ("sorted", 6), ("syn", 2), ("latest", 1), ("bins", 3)])
@pytest.mark.parametrize("mode", [0, 2])
def test_double_exponential_synapse_forward_backward(kind, cap, mode):
    """Double-exponential synapse (Section 3.2, closing remark): two synaptic states take every
    jump, the membrane integrates their difference; the weight gathers the sum of their adjoints,
    the delay (and, in the spike-time mode, the emitting spike) each adjoint over its own time
    constant.  Whole-step delays."""
    wl = synth.ragged_network(150, 300, 30, seed=15, rate_hz=250.0, t=160, b=2, w_mean=0.003, w_std=0.003)
    wl.tau_syn_ms, wl.tau_rise_ms = 1.7, 0.5
    ref = _compare_backward(wl, KINDS[kind], cap, 160, 2, surrogate=mode, tape_spike_capacity=2 * 160 * 150)
    assert ref.spikes.sum() > 100
    one = oracle.Run(synth.Workload(**{**wl.__dict__, "tau_rise_ms": 0.0}), KINDS[kind], cap, n_steps=160, batch=2)
    assert not np.array_equal(one.U, ref.U)      # the second state changes the dynamics
    if kind != "ring":
        assert ref.counters()["dropped"] > 0


def test_double_exponential_synapse_needs_whole_step_delays():
    wl = synth.ragged_network(20, 10, 10, seed=3, continuous=True)
    wl.tau_syn_ms, wl.tau_rise_ms = 1.7, 0.5
    with pytest.raises(adseq.AdseqError):
        adseq.Adseq(wl, adseq.RING)


@pytest.mark.parametrize("kind,cap", [("ring", 0), ("fifo", 32), ("fifo", 2), ("sorted", 128), ("syn", 4)])
def test_cfg1_forward_backward(kind, cap):
    """Config 1 (1,000 neurons, fan-out 100, batch 16, 2,000 steps), MSE spike-count loss."""
    wl = synth.cfg1()
    ref = _compare_backward(wl, KINDS[kind], cap, wl.n_steps, wl.batch, use_dU=False)
    if cap == 2:
        assert ref.counters()["dropped"] > 10000
    else:
        assert ref.counters()["dropped"] == 0


@pytest.mark.parametrize("kind,cap", [("ring", 0), ("fifo", 3), ("sorted", 3)])
def test_spike_counts_match_the_raster(kind, cap):
    wl = synth.ragged_network(300, 200, 30, seed=6, rate_hz=250.0, t=130, b=3, w_mean=0.01, w_std=0.01)
    ref = oracle.Run(wl, KINDS[kind], cap, n_steps=130, batch=3)
    sim, _ = H.run_gpu(wl, KINDS[kind], cap, n_steps=130, batch=3, per_step=False)
    counts = torch.full((3 * 300,), -5, dtype=torch.int32, device=sim.dev)
    sim.spike_counts(counts)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(counts.cpu().numpy().reshape(3, 300), ref.spikes.sum(axis=0))
    assert ref.spikes.sum() > 100
    sim.close()


def test_backward_without_tape_is_refused():
    wl = synth.cfg0()
    sim = adseq.Adseq(wl, adseq.RING, record_tape=False)
    sim.run(0, 10)
    g = torch.zeros(wl.n_synapses, device=sim.dev)
    with pytest.raises(adseq.AdseqError) as ei:
        sim.backward(None, None, g, g.clone())
    assert ei.value.code == -5
    sim.close()


def test_tape_overflow_is_reported():
    wl = synth.cfg0(seed=11)
    wl.ext_rate_hz = 400.0
    sim = adseq.Adseq(wl, adseq.FIFO, 4, record_tape=True, max_steps=200, tape_spike_capacity=5)
    sim.run(0, 200)
    with pytest.raises(adseq.AdseqError) as ei:
        sim.drop_count()
    assert ei.value.code == -7
    sim.close()


# ---------------------------------------------------------------- the larger configs, shortened

@pytest.mark.parametrize("kind,cap", [("ring", 0), ("fifo", 8), ("fifo", 32)])
def test_cfg2_shape_forward(kind, cap):
    """Config 2's network (10,000 neurons, fan-out 1,000, delays 1..200) for 240 steps with a
    drive strong enough to make it fire within them; bounded kinds overflow heavily."""
    wl = synth.cfg2(rate_hz=100.0)
    ref, _ = _compare_forward(wl, KINDS[kind], cap, T=240, check_sets=False)
    assert ref.spikes.sum() > 2000
    if kind != "ring":
        assert ref.counters()["dropped"] > 1000000


@pytest.mark.parametrize("kind,cap", [("sorted", 128), ("fifo", 32), ("ring", 0)])
def test_cfg4_shape_forward_backward(kind, cap):
    """Config 4's network (4,096 neurons, fan-out 256, lognormal weights with 20 % inhibitory
    sources, continuous delays 0.1..20 ms), 6 trials, 300 steps, delay and weight gradients."""
    wl = synth.cfg4(n_steps=300, batch=6)
    wl.ext_rate_hz = 250.0
    ref = _compare_backward(wl, KINDS[kind], cap, 300, 6, use_dU=False,
                            tape_spike_capacity=300 * 6 * 4096 // 4)
    assert ref.spikes.sum() > 3000


@pytest.mark.parametrize("kind,cap", [("ring", 0), ("fifo", 4)])
def test_library_kernel_timing_counts_its_launches(kind, cap):
    """adseq_profile / adseq_profile_read: per kernel class, the launches of a run and times that
    are positive and add up to less than the run took; the results of the run are unchanged."""
    import time
    wl = synth.ragged_network(300, 200, 40, seed=8, rate_hz=250.0, t=100, b=2, w_mean=0.01, w_std=0.01)
    T = 100
    ref = oracle.Run(wl, KINDS[kind], cap, n_steps=T, batch=2)
    sim = adseq.Adseq(wl, KINDS[kind], cap, batch=2, record_tape=True, max_steps=T)
    sim.profile(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    sim.run(0, T)
    g_w = torch.empty(wl.n_synapses, device=sim.dev)
    g_d = torch.empty(wl.n_synapses, device=sim.dev)
    sim.backward(torch.full((2 * wl.n_neurons,), 1e-3, device=sim.dev), None, g_w, g_d)
    p = sim.profile_read()
    wall_ms = (time.perf_counter() - t0) * 1e3
    np.testing.assert_array_equal(sim.tape()["U"].cpu().numpy().view(np.uint32), ref.U.view(np.uint32))
    assert p["lif"]["launches"] == T and p["bwd_neurons"]["launches"] == T
    if kind == "ring":      # one expansion and one far gather per window boundary inside the run
        # (the reverse sweep goes window by window: every window, the first included, ends with a gather)
        assert p["fan_out"]["launches"] == (T - 1) // 16 and p["bwd_gather"]["launches"] == (T - 1) // 16 + 1
    else:                   # one fan-out per step; a reverse gather for every step that has spikes
        assert p["fan_out"]["launches"] == T and 0 < p["bwd_gather"]["launches"] <= T
    total = sum(v["ms"] for v in p.values())
    assert all(v["ms"] > 0 for v in p.values()) and total < wall_ms
    again = sim.profile_read()                      # read and forgotten
    assert all(v["launches"] == 0 for v in again.values())
    sim.profile(False)
    sim.close()
