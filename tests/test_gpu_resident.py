"""The ring's resident step kernels (adseq_run: all the steps of a window in one launch on the
blocks of one XCD, ring_resident.h) against the CPU oracle, through the C ABI: membrane trace bit
for bit, counters, spike counts; every register layout (1, 4, 8 neurons per thread), several
window lengths, batches, the synaptic current states, runs cut into pieces and mixed with single
steps, resets, and agreement with the one-launch-per-step path; likewise the forward kernel over the
whole chip (ring_resident_forward.h) and the two resident reverse kernels -- without a grid barrier
(ring_flow_reverse.h, the default) and with one (ring_resident_reverse.h) -- with their layouts of
one, four and eight neurons per thread, block counts, spreads over the XCDs and failure paths."""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2512_05906_amd import adseq, synth
from tests import helpers as H

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _resident_on(monkeypatch):
    """By default the resident kernels run up to 32,768 state cells; here wherever the layout allows."""
    monkeypatch.setenv("ADSEQ_RING_RESIDENT", "1")


@pytest.fixture(params=["flow", "barrier"])
def rev_kernel(request, monkeypatch):
    """The two resident reverse kernels: blocks that wait for the cells they gather (the default) and a grid
    barrier per step."""
    monkeypatch.setenv("ADSEQ_RING_REVERSE_FLOW", "1" if request.param == "flow" else "0")
    return request.param


def _run_pieces(wl, T, B, pieces, **kw):
    """Forward run through adseq_run / adseq_step in the given pieces (int = that many steps in one
    adseq_run call, 's' = one adseq_step call); returns (sim, U, counters, counts)."""
    sim = adseq.Adseq(wl, adseq.RING, 0, batch=B, record_tape=True, max_steps=T, **kw)
    n = 0
    for p in pieces:
        if p == "s":
            sim.step(n); n += 1
        else:
            sim.run(n, p); n += p
    assert n == T
    torch.cuda.synchronize()
    U = sim.tape()["U"].cpu().numpy().copy()
    counts = torch.empty(B * wl.n_neurons, dtype=torch.int32, device=sim.dev)
    sim.spike_counts(counts)
    return sim, U, sim.counters(), counts.cpu().numpy()


def _check(wl, T, B, pieces, **kw):
    ref = oracle.Run(wl, oracle.RING, 0, n_steps=T, batch=B, n_threads=8)
    sim, U, c, counts = _run_pieces(wl, T, B, pieces, **kw)
    np.testing.assert_array_equal(U.view(np.uint32), ref.U.view(np.uint32))
    rc = ref.counters()
    for key in ("enqueued", "dropped", "delivered", "sum_enqueued", "sum_dropped", "sum_delivered"):
        assert c[key] == rc[key], key
    assert c["error_bits"] == 0
    np.testing.assert_array_equal(counts.reshape(B, -1), ref.spikes.sum(axis=0))
    sim.close()
    return ref


@pytest.mark.parametrize("n,fan,b", [(100, 30, 1), (301, 200, 3), (2500, 60, 16), (40000, 20, 1), (5000, 30, 20), (9000, 30, 20)])
def test_resident_forward_sizes(n, fan, b):
    """1, 2 and 4 groups of four neurons per thread; rows that are and are not 16-byte aligned; one block to
    32 blocks; one trial and many; and a state array beyond the resident kernels (a launch per step)."""
    wl = synth.ragged_network(n, fan, 40, seed=n + b, rate_hz=700.0, t=120, b=b, w_mean=0.6 / fan, w_std=0.4 / fan)
    ref = _check(wl, 120, b, [120])
    assert ref.spikes.sum() > 100


@pytest.mark.parametrize("window", [2, 8, 16, 64])
def test_resident_window_lengths_and_pieces(window, monkeypatch):
    monkeypatch.setenv("ADSEQ_RING_WINDOW", str(window))
    wl = synth.ragged_network(700, 300, 37, seed=5, rate_hz=300.0, t=150, b=2, w_mean=0.004, w_std=0.003)
    ref = _check(wl, 150, 2, [1, 30, "s", "s", 7, 64, "s", 45])
    assert ref.spikes.sum() > 300


@pytest.mark.parametrize("tau_syn,tau_rise", [(5.0, 0.0), (5.0, 1.0)])
def test_resident_synaptic_states(tau_syn, tau_rise):
    wl = synth.ragged_network(400, 150, 30, seed=8, rate_hz=250.0, t=140, b=2, w_mean=0.004, w_std=0.003)
    wl.tau_syn_ms, wl.tau_rise_ms = tau_syn, tau_rise
    ref = _check(wl, 140, 2, [50, "s", 89])
    assert ref.spikes.sum() > 100


def test_resident_matches_step_launches(monkeypatch):
    """The same run with the resident kernels switched off: identical trace and counters."""
    wl = synth.ragged_network(5000, 80, 50, seed=12, rate_hz=200.0, t=100, b=4, w_mean=0.008, w_std=0.006)
    sim, U1, c1, n1 = _run_pieces(wl, 100, 4, [100])
    sim.close()
    monkeypatch.setenv("ADSEQ_RING_RESIDENT", "0")
    sim, U0, c0, n0 = _run_pieces(wl, 100, 4, [100])
    sim.close()
    np.testing.assert_array_equal(U1.view(np.uint32), U0.view(np.uint32))
    assert c1 == c0 and c1["tape_spikes"] > 500
    np.testing.assert_array_equal(n1, n0)


def test_resident_reset_and_rerun():
    wl = synth.ragged_network(1200, 100, 20, seed=3, rate_hz=200.0, t=90, b=2, w_mean=0.006, w_std=0.004)
    sim, U1, c1, _ = _run_pieces(wl, 90, 2, [90])
    sim.reset()
    sim.run(0, 40); sim.run(40, 50)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(sim.tape()["U"].cpu().numpy().view(np.uint32), U1.view(np.uint32))
    assert sim.counters() == c1
    sim.close()


@pytest.mark.parametrize("resident", ["0", "1"])
def test_ring_popped_sum_is_counted(resident, monkeypatch):
    """The ring derives its delivered counters from the spikes (offered minus still in flight).
    With ADSEQ_RING_COUNT_POPPED = 1 the step kernels add up, cell by cell, the Q8.24 values they
    pop, and sum_delivered is that count: it must equal the oracle's sum over delivered events
    (a lost or doubled add anywhere in the scatter or the window expansion would show), and the
    derived figure must agree with it."""
    wl = synth.ragged_network(3000, 120, 45, seed=17, rate_hz=300.0, t=160, b=2, w_mean=0.005, w_std=0.004)
    ref = oracle.Run(wl, oracle.RING, 0, n_steps=160, batch=2, n_threads=2)
    monkeypatch.setenv("ADSEQ_RING_RESIDENT", resident)
    _, _, derived, _ = _run_pieces(wl, 160, 2, [70, "s", 89])
    monkeypatch.setenv("ADSEQ_RING_COUNT_POPPED", "1")
    _, _, counted, _ = _run_pieces(wl, 160, 2, [70, "s", 89])
    assert counted["sum_delivered"] == ref.counters()["sum_delivered"] == derived["sum_delivered"]
    assert counted["sum_delivered"] != 0 and counted["delivered"] == ref.counters()["delivered"]


@pytest.mark.parametrize("margin", ["20", "0", "100000"])
@pytest.mark.parametrize("n,fan,b", [(100, 30, 1), (301, 200, 4), (2500, 60, 16), (40000, 20, 1), (131072, 6, 1)])
def test_forward_chip_sizes_and_margins(n, fan, b, margin, monkeypatch):
    """The forward kernel over the whole chip that requests the rows of the neurons about to spike ahead of the
    barrier (ring_resident_forward.h; ADSEQ_RING_FORWARD_CHIP=1): membrane trace bit for bit, counters, spike counts.
    One block to 128; a trial boundary inside a thread's neurons; the default margin, margin 0 (a neuron lifted over the
    threshold by the last step's events was no candidate: the slow way) and a margin that makes every neuron a
    candidate (only the first 32 of a block are requested ahead, the others go the slow way)."""
    monkeypatch.setenv("ADSEQ_RING_FORWARD_CHIP", "1")
    monkeypatch.setenv("ADSEQ_RING_FORWARD_MARGIN", margin)
    wl = synth.ragged_network(n, fan, 40, seed=n + b, rate_hz=700.0, t=120, b=b, w_mean=0.6 / fan, w_std=0.4 / fan)
    ref = _check(wl, 120, b, [120])
    assert ref.spikes.sum() > 100


@pytest.mark.parametrize("window", [2, 8, 64])
def test_forward_chip_window_lengths_and_pieces(window, monkeypatch):
    monkeypatch.setenv("ADSEQ_RING_FORWARD_CHIP", "1")
    monkeypatch.setenv("ADSEQ_RING_WINDOW", str(window))
    wl = synth.ragged_network(700, 300, 37, seed=5, rate_hz=300.0, t=150, b=2, w_mean=0.004, w_std=0.003)
    ref = _check(wl, 150, 2, [1, 30, "s", "s", 7, 64, "s", 45])
    assert ref.spikes.sum() > 300
    # delays of one and two steps only: rows with more than 64 entries inside the window
    wl = synth.ragged_network(900, 200, 2, seed=6, rate_hz=400.0, t=70, b=2, w_mean=0.004, w_std=0.004)
    _check(wl, 70, 2, [70])


@pytest.mark.parametrize("surrogate", [adseq.SURR_SUPERSPIKE, adseq.GRAD_SPIKE_TIME])
@pytest.mark.parametrize("n,b,T", [(700, 3, 150), (6000, 2, 100)])
def test_reverse_sweep_by_windows(surrogate, n, b, T, monkeypatch):
    """The ring's reverse sweep one window at a time (a dense pass per neuron, the near
    corrections of the window's spikes step by step inside one workgroup, then the far gather;
    by default only for up to 1,024 state cells, here forced on): both gradients against the
    oracle, with a cotangent on the membrane values as well, in both gradient modes, a run length
    that is not a multiple of the window, and agreement with the sweep of one launch per step."""
    wl = synth.ragged_network(n, 200, 40, seed=n, rate_hz=400.0, t=T, b=b, w_mean=0.004, w_std=0.004)
    ref = oracle.Run(wl, oracle.RING, 0, n_steps=T, batch=b, surrogate=surrogate, n_threads=4)
    assert ref.spikes.sum() > 300
    rng = np.random.default_rng(n)
    dc = rng.normal(0, 1e-3, (b, n)).astype(np.float32)
    dU = rng.normal(0, 1e-4, (T, b, n)).astype(np.float32)
    gw, gd = ref.backward(dc, dU)
    got = {}
    for mode in ("1", "0"):
        monkeypatch.setenv("ADSEQ_RING_REVERSE_WINDOWS", mode)
        sim = adseq.Adseq(wl, adseq.RING, 0, batch=b, record_tape=True, max_steps=T, surrogate=surrogate)
        sim.run(0, T)
        g_w = torch.empty(wl.n_synapses, device=sim.dev)
        g_d = torch.empty(wl.n_synapses, device=sim.dev)
        sim.backward(torch.from_numpy(dc).to(sim.dev), torch.from_numpy(dU).to(sim.dev), g_w, g_d)
        torch.cuda.synchronize()
        assert sim.counters()["error_bits"] == 0
        got[mode] = (g_w.cpu().numpy(), g_d.cpu().numpy())
        H.grad_close(got[mode][0], gw)
        H.grad_close(got[mode][1], gd)
        sim.close()
    H.grad_close(got["1"][0], got["0"][0])
    H.grad_close(got["1"][1], got["0"][1])


@pytest.mark.parametrize("surrogate", [adseq.SURR_SUPERSPIKE, adseq.GRAD_SPIKE_TIME])
@pytest.mark.parametrize("n,b,T,d_max,rate,continuous", [(700, 3, 150, 40, 400.0, False), (6000, 2, 100, 40, 2500.0, False),
                                                        (20000, 4, 70, 40, 400.0, False), (900, 4, 70, 2, 400.0, False),
                                                        (1500, 2, 90, 30, 400.0, True)])
def test_resident_reverse_sweep(surrogate, n, b, T, d_max, rate, continuous, rev_kernel, monkeypatch):
    """The reverse steps of a window in one launch with a grid barrier per step (ring_resident_reverse.h):
    both gradients against the oracle, with a cotangent on the membrane values as well, in both
    gradient modes; a few blocks and 128; a run length that is not a multiple of the
    window; a drive under which a block has more than 32 spikes in a step (the spikes beyond a
    wavefront's first batch); delays of one and two steps only (rows of up to 200 entries: more than
    64 inside the window, the gathers beyond a wavefront's first load); continuous delays; and
    agreement with the sweep of one launch per step."""
    wl = synth.ragged_network(n, 200, d_max, seed=n, rate_hz=rate, t=T, b=b, w_mean=0.004, w_std=0.004,
                              continuous=continuous)
    ref = oracle.Run(wl, oracle.RING, 0, n_steps=T, batch=b, surrogate=surrogate, n_threads=4)
    assert ref.spikes.sum() > 300
    rng = np.random.default_rng(n)
    dc = rng.normal(0, 1e-3, (b, n)).astype(np.float32)
    dU = rng.normal(0, 1e-4, (T, b, n)).astype(np.float32)
    gw, gd = ref.backward(dc, dU)
    got = {}
    monkeypatch.setenv("ADSEQ_RING_REVERSE_WINDOWS", "0")
    for mode in ("1", "0"):
        monkeypatch.setenv("ADSEQ_RING_RESIDENT_REVERSE", mode)
        sim = adseq.Adseq(wl, adseq.RING, 0, batch=b, record_tape=True, max_steps=T, surrogate=surrogate)
        sim.run(0, T)
        g_w = torch.empty(wl.n_synapses, device=sim.dev)
        g_d = torch.empty(wl.n_synapses, device=sim.dev)
        sim.backward(torch.from_numpy(dc).to(sim.dev), torch.from_numpy(dU).to(sim.dev), g_w, g_d)
        torch.cuda.synchronize()
        assert sim.counters()["error_bits"] == 0
        got[mode] = (g_w.cpu().numpy(), g_d.cpu().numpy())
        H.grad_close(got[mode][0], gw)
        H.grad_close(got[mode][1], gd)
        # a second sweep over the same tape gives the same gradients (carry, window and far terms start from zero again)
        if mode == "1":
            sim.backward(torch.from_numpy(dc).to(sim.dev), torch.from_numpy(dU).to(sim.dev), g_w, g_d)
            torch.cuda.synchronize()
            H.grad_close(g_w.cpu().numpy(), gw)
        sim.close()
    H.grad_close(got["1"][0], got["0"][0])
    H.grad_close(got["1"][1], got["0"][1])


def _reverse_against_oracle(wl, T, b, surrogate=adseq.SURR_SUPERSPIKE):
    ref = oracle.Run(wl, oracle.RING, 0, n_steps=T, batch=b, surrogate=surrogate, n_threads=4)
    rng = np.random.default_rng(wl.n_neurons)
    dc = rng.normal(0, 1e-3, (b, wl.n_neurons)).astype(np.float32)
    gw, gd = ref.backward(dc, None)
    sim = adseq.Adseq(wl, adseq.RING, 0, batch=b, record_tape=True, max_steps=T, surrogate=surrogate)
    sim.run(0, T)
    g_w = torch.empty(wl.n_synapses, device=sim.dev)
    g_d = torch.empty(wl.n_synapses, device=sim.dev)
    sim.backward(torch.from_numpy(dc).to(sim.dev), None, g_w, g_d)
    torch.cuda.synchronize()
    assert sim.counters()["error_bits"] == 0
    H.grad_close(g_w.cpu().numpy(), gw)
    H.grad_close(g_d.cpu().numpy(), gd)
    sim.close()
    return ref


@pytest.mark.parametrize("blocks,stride", [("8", "8"), ("32", "1"), ("256", "2"), ("128", "4")])
def test_resident_reverse_block_counts_and_spread(blocks, stride, rev_kernel, monkeypatch):
    """The resident reverse kernel with few and many taking-part blocks, on one XCD and spread over
    all of them (every stride-th block of the grid takes part): nothing in its results depends on
    where the blocks run.  A trial boundary inside a thread's four neurons (N = 301, four trials), no
    cotangent on the membrane values, windows of 8 steps."""
    monkeypatch.setenv("ADSEQ_RING_REVERSE_WINDOWS", "0")
    monkeypatch.setenv("ADSEQ_RING_RESIDENT_REVERSE", "1")
    monkeypatch.setenv("ADSEQ_RING_REVERSE_BLOCKS", blocks)
    monkeypatch.setenv("ADSEQ_RING_RESIDENT_STRIDE", stride)
    monkeypatch.setenv("ADSEQ_RING_WINDOW", "8")
    wl = synth.ragged_network(301, 150, 30, seed=41, rate_hz=500.0, t=90, b=4, w_mean=0.006, w_std=0.004)
    ref = _reverse_against_oracle(wl, 90, 4)
    assert ref.spikes.sum() > 300
    wl = synth.ragged_network(30000, 40, 30, seed=42, rate_hz=500.0, t=50, b=2, w_mean=0.02, w_std=0.01)
    ref = _reverse_against_oracle(wl, 50, 2, adseq.GRAD_SPIKE_TIME)
    assert ref.spikes.sum() > 300


def test_resident_reverse_falls_back_where_the_layout_does_not_fit(rev_kernel, monkeypatch):
    """B N not a multiple of 4 (rows of the window not 16-byte aligned): the reverse sweep goes by one launch per step,
    same gradients.  More state cells than the blocks hold at four neurons per thread (8 blocks of 2,048 < 20,000): the
    kernel with a grid barrier falls back likewise, the one without takes eight neurons per thread."""
    monkeypatch.setenv("ADSEQ_RING_REVERSE_WINDOWS", "0")
    wl = synth.ragged_network(1201, 100, 30, seed=43, rate_hz=500.0, t=60, b=3, w_mean=0.008, w_std=0.005)
    _reverse_against_oracle(wl, 60, 3)
    monkeypatch.setenv("ADSEQ_RING_REVERSE_BLOCKS", "8")
    wl = synth.ragged_network(20000, 40, 30, seed=44, rate_hz=500.0, t=40, b=1, w_mean=0.02, w_std=0.01)   # 8 blocks of 2,048 < 20,000
    _reverse_against_oracle(wl, 40, 1)


def test_resident_kernels_need_their_blocks_on_the_chip_together(monkeypatch):
    """The grid barrier needs all blocks of a launch resident at once.  A device that cannot hold them (here: the
    host check is told of 64 compute units) gets one launch per time step, forward and in reverse, and the same
    results; with the real count the windows go by one launch each."""
    wl = synth.ragged_network(6000, 40, 30, seed=47, rate_hz=600.0, t=64, b=2, w_mean=0.02, w_std=0.01)

    def launches():
        sim = adseq.Adseq(wl, adseq.RING, 0, batch=2, record_tape=True, max_steps=64)
        sim.profile(True)
        sim.run(0, 64)
        g = torch.empty(wl.n_synapses, device=sim.dev)
        sim.backward(torch.zeros(2 * 6000, device=sim.dev) + 1e-3, None, g, g.clone())
        torch.cuda.synchronize()
        p = sim.profile_read()
        assert sim.counters()["error_bits"] == 0
        sim.close()
        return p["lif"]["launches"], p["bwd_neurons"]["launches"]

    fwd, rev = launches()
    assert fwd < 64 and rev < 64
    monkeypatch.setenv("ADSEQ_RING_ASSUME_CUS", "64")
    fwd, rev = launches()
    assert fwd == 64 and rev == 64
    _check(wl, 64, 2, [64])
    _reverse_against_oracle(wl, 64, 2)


def test_resident_reverse_wait_that_runs_out_is_reported(rev_kernel, monkeypatch):
    """Failure path of the reverse kernels' bounded waits, forced from the host (one poll per wait at the grid barrier;
    without a barrier, spiking neurons that withhold their final adjoints and 16 polls per wait): every kernel
    runs to its end, the error word carries bit 32 after the sweep, a reset clears it, and a handle with the
    ordinary limit gives the oracle's gradients."""
    monkeypatch.setenv("ADSEQ_RING_REVERSE_WINDOWS", "0")
    monkeypatch.setenv("ADSEQ_RING_RESIDENT", "0")
    monkeypatch.setenv("ADSEQ_RING_FORWARD_CHIP", "0")   # (the forward run by one launch per step: no wait of its own to run out)
    monkeypatch.setenv("ADSEQ_RING_REVERSE_DELAY", "0")
    wl = synth.ragged_network(40000, 30, 20, seed=45, rate_hz=700.0, t=60, b=2, w_mean=0.02, w_std=0.01)
    sim = adseq.Adseq(wl, adseq.RING, 0, record_tape=True, max_steps=60)
    sim.run(0, 60)
    torch.cuda.synchronize()
    assert sim.counters()["error_bits"] == 0
    sim.close()
    monkeypatch.setenv("ADSEQ_RING_RESIDENT_SPINS", "16" if rev_kernel == "flow" else "1")
    if rev_kernel == "flow":
        monkeypatch.setenv("ADSEQ_RING_FLOW_WITHHOLD", "1")
    sim = adseq.Adseq(wl, adseq.RING, 0, record_tape=True, max_steps=60)
    sim.run(0, 60)
    g = torch.empty(wl.n_synapses, device=sim.dev)
    sim.backward(torch.zeros(2 * 40000, device=sim.dev) + 1e-3, None, g, g.clone())
    torch.cuda.synchronize()
    assert sim.counters()["error_bits"] & 32
    with pytest.raises(adseq.AdseqError):
        sim.drop_count()
    sim.reset()
    assert sim.counters()["error_bits"] == 0
    sim.close()
    monkeypatch.delenv("ADSEQ_RING_RESIDENT_SPINS")
    monkeypatch.delenv("ADSEQ_RING_REVERSE_DELAY")
    monkeypatch.delenv("ADSEQ_RING_FLOW_WITHHOLD", raising=False)
    _reverse_against_oracle(wl, 60, 2)


def test_forward_chip_wait_that_runs_out_is_reported(monkeypatch):
    """The same for the forward kernel over the whole chip: one poll per wait, no delay before it; the kernels run
    to their end, the error word carries bit 32, adseq_drop_count and adseq_backward refuse the run, a reset clears it."""
    monkeypatch.setenv("ADSEQ_RING_FORWARD_CHIP", "1")
    monkeypatch.setenv("ADSEQ_RING_REVERSE_DELAY", "0")
    monkeypatch.setenv("ADSEQ_RING_RESIDENT_SPINS", "1")
    wl = synth.ragged_network(40000, 30, 20, seed=46, rate_hz=700.0, t=60, b=2, w_mean=0.02, w_std=0.01)
    sim = adseq.Adseq(wl, adseq.RING, 0, record_tape=True, max_steps=60)
    sim.run(0, 60)
    torch.cuda.synchronize()
    assert sim.counters()["error_bits"] & 32
    with pytest.raises(adseq.AdseqError):
        sim.drop_count()
    g = torch.empty(wl.n_synapses, device=sim.dev)
    with pytest.raises(adseq.AdseqError):
        sim.backward(torch.zeros(2 * 40000, device=sim.dev), None, g, g.clone())
    sim.reset()
    assert sim.counters()["error_bits"] == 0
    sim.close()
    monkeypatch.delenv("ADSEQ_RING_RESIDENT_SPINS")
    monkeypatch.delenv("ADSEQ_RING_REVERSE_DELAY")
    ref = _check(wl, 60, 2, [60])
    assert ref.spikes.sum() > 100


def test_range_warning_for_sums_that_could_wrap():
    """adseq_create adds up |amplitude| over every target's incoming synapses; where that reaches
    128 (the range of the Q8.24 sums) the counters carry the warning bit 64, also after a reset."""
    wl = synth.ragged_network(50, 40, 10, seed=2, rate_hz=100.0, t=20, b=1, w_mean=0.05, w_std=0.01)
    sim = adseq.Adseq(wl, adseq.RING, 0)
    assert sim.counters()["error_bits"] == 0
    sim.close()
    big = synth.ragged_network(50, 40, 10, seed=2, rate_hz=100.0, t=20, b=1, w_mean=9.0, w_std=0.5)
    for kind, cap in ((adseq.RING, 0), (adseq.FIFO, 4)):
        sim = adseq.Adseq(big, kind, cap)
        assert sim.counters()["error_bits"] == 64
        sim.reset()
        sim.run(0, 5)
        assert sim.counters()["error_bits"] & 64
        sim.close()


def test_resident_wait_that_runs_out_is_reported(monkeypatch):
    """Failure path of the resident kernels' bounded waits, forced from the host: with a limit of
    one poll per wait (ADSEQ_RING_RESIDENT_SPINS=1) the 32 blocks do not wait for one another, every
    kernel still runs to its end, the error word carries bit 32, and adseq_drop_count and
    adseq_backward refuse the run; a reset clears the state, and a handle with the ordinary limit
    gives the oracle's result on the same network."""
    wl = synth.ragged_network(5000, 30, 20, seed=21, rate_hz=700.0, t=60, b=20, w_mean=0.02, w_std=0.01)
    monkeypatch.setenv("ADSEQ_RING_RESIDENT_SPINS", "1")
    sim = adseq.Adseq(wl, adseq.RING, 0, record_tape=True, max_steps=60)
    sim.run(0, 60)
    torch.cuda.synchronize()
    assert sim.counters()["error_bits"] & 32
    with pytest.raises(adseq.AdseqError):
        sim.drop_count()
    g = torch.empty(wl.n_synapses, device=sim.dev)
    with pytest.raises(adseq.AdseqError):
        sim.backward(torch.zeros(20 * 5000, device=sim.dev), None, g, g.clone())
    sim.reset()
    assert sim.counters()["error_bits"] == 0
    sim.close()
    monkeypatch.delenv("ADSEQ_RING_RESIDENT_SPINS")
    ref = _check(wl, 60, 20, [60])
    assert ref.spikes.sum() > 100
