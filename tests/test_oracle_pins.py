"""Pins of the CPU oracle against things other than itself: brute force,
closed forms, invariants, library routines, published test vectors."""
import math
import os

import numpy as np
import pytest
import scipy.sparse as sp

from oracle import brute, oracle, tangent
from paper_2512_05906_amd import synth


def _src(wl):
    return np.repeat(np.arange(wl.n_neurons), np.diff(wl.row_ptr))


# ---------------------------------------------------------------- hash / helpers

def test_mix64_matches_published_splitmix64_vectors():
    # first outputs of SplitMix64 seeded with 1234567 (reference vectors of the
    # public-domain generator by S. Vigna)
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "splitmix64_seed1234567.txt")
    want = [int(l) for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(want) == 5
    s = 1234567
    for w in want:
        s = (s + 0x9E3779B97F4A7C15) & (2**64 - 1)
        assert oracle.mix64(s) == w


def test_drive_rate_matches_bernoulli_probability():
    p = 50.0 * np.float32(0.1) * 1e-3
    thr = math.floor(float(p) * 2**32)
    hits = sum(oracle.drive_bits(7, g, n) < thr for g in range(200) for n in range(1000))
    n = 200 * 1000
    assert abs(hits - n * p) < 5 * math.sqrt(n * p)


def test_exp_neg_taylor_vs_libm():
    for x in np.linspace(0.0, 1.0, 101):
        assert abs(oracle.exp_neg(float(x)) - math.exp(-x)) < 4e-16


# ---------------------------------------------------------------- LIF closed form

def test_lif_charging_curve_closed_form():
    """One neuron, constant current, no synapses: U[n] = I (1 - a^(n+1)) / (1 - a)
    until the first spike (geometric series of the leaky update)."""
    wl = synth.Workload("one", 1, 0, 400, 1, 1, ext_rate_hz=0.0,
                        row_ptr=np.zeros(2, np.int64), col=np.zeros(0, np.int32),
                        weight=np.zeros(0, np.float32), delay_steps=np.zeros(0, np.uint8))
    I0 = 0.006
    i_ext = np.full((400, 1, 1), I0, np.float32)
    r = oracle.Run(wl, oracle.RING, i_ext=i_ext)
    U, S = r.U[:, 0, 0], r.spikes[:, 0, 0]
    alpha = math.exp(-float(np.float32(0.1)) / 20.0)
    first = int(np.argmax(S)) if S.any() else len(S)
    assert first > 100  # I0/(1-alpha) = 1.2 > 1 so it does fire, but late
    n = np.arange(first + 1)
    closed = float(np.float32(I0)) * (1 - alpha ** (n + 1)) / (1 - alpha)
    np.testing.assert_allclose(U[:first + 1], closed, rtol=2e-5)
    assert S[first] == 1 and closed[first] >= 1.0 - 1e-4
    # reset to 0: the next value restarts the curve
    np.testing.assert_allclose(U[first + 1], closed[0], rtol=1e-6)


# ---------------------------------------------------------------- delivery definition

@pytest.mark.parametrize("kind,cap", [(oracle.RING, 0), (oracle.SORTED, 4096), (oracle.FIFO, 4096)])
def test_currents_equal_brute_force_cfg0(kind, cap):
    wl = synth.cfg0()
    r = oracle.Run(wl, kind, cap, keep_currents=True, log_events=True)
    S = r.spikes[:, 0, :]
    assert 100 < S.sum() < 20000
    amp = wl.weight.astype(np.float64)
    I = brute.delivered_currents(S, wl.row_ptr, wl.col, amp, wl.delay_steps)
    got = r.Iq[:, 0, :].astype(np.float64) / 2**24
    # fixed point resolution 2^-25 per event, a few events per (neuron, step)
    np.testing.assert_allclose(got, I, rtol=0, atol=1e-6)
    assert r.counters()["dropped"] == 0


def test_unit_delay_reduces_to_sparse_matvec():
    """All delays one step: I[n+1] = W^T s[n] (scipy CSR product)."""
    wl = synth.cfg0(seed=5)
    wl.delay_steps[:] = 1
    r = oracle.Run(wl, oracle.RING, keep_currents=True)
    S = r.spikes[:, 0, :].astype(np.float64)
    aq = r.a_q.astype(np.float64)
    W = sp.csr_matrix((aq, wl.col, wl.row_ptr), shape=(wl.n_neurons, wl.n_neurons))
    want = (W.T @ S[:-1].T).T
    np.testing.assert_array_equal(r.Iq[1:, 0, :].astype(np.float64), want)
    assert not r.Iq[0].any()


def test_quantised_amplitudes():
    wl = synth.cfg0()
    wl.weight[:4] = [0.1, -0.1, 200.0, -200.0]
    r = oracle.Run(wl, oracle.RING, n_steps=1)
    aq = r.a_q
    assert aq[0] == int(np.rint(np.float64(np.float32(0.1)) * 2**24))
    assert aq[1] == -aq[0]
    assert aq[2] == 2**31 - 1 and aq[3] == -2**31   # saturates at +-128


@pytest.mark.parametrize("kind,cap", [(oracle.RING, 0), (oracle.FIFO, 3), (oracle.SORTED, 5)])
def test_every_admitted_event_delivered_exactly_once(kind, cap):
    wl = synth.cfg0(seed=11)
    wl.ext_rate_hz = 120.0
    r = oracle.Run(wl, kind, cap, log_events=True, keep_currents=True)
    S = r.spikes[:, 0, :]
    T = wl.n_steps
    D = wl.delay_steps.astype(np.int64)
    # emitted events from the raster
    emitted = set()
    for n, i in zip(*np.nonzero(S)):
        for p in range(wl.row_ptr[i], wl.row_ptr[i + 1]):
            emitted.add((p, int(n), int(n + D[p])))
    dl, dr = r.event_log("delivered"), r.event_log("dropped")
    delivered = list(zip(dl["syn"].tolist(), dl["n_emit"].tolist(), dl["k"].tolist()))
    dropped = list(zip(dr["syn"].tolist(), dr["n_emit"].tolist(), dr["k"].tolist()))
    assert len(set(delivered)) == len(delivered)            # at most once
    assert set(delivered) <= emitted and set(dropped) <= emitted
    assert not (set(delivered) & set(dropped))
    in_run = {e for e in emitted if e[2] < T} - set(dropped)
    assert set(delivered) == in_run                          # exactly once, at n + D
    c = r.counters()
    assert c["enqueued"] == len(emitted)
    assert c["enqueued"] == c["delivered"] + c["dropped"] + c["in_flight"]
    assert c["sum_enqueued"] == c["sum_delivered"] + c["sum_dropped"] + c["sum_in_flight"]
    if kind == oracle.RING:
        assert c["dropped"] == 0
    else:
        assert c["dropped"] > 0 and c["max_occupancy"] == cap
    # the popped sums are exactly the delivered amplitudes
    aq = r.a_q.astype(np.int64)
    tot = np.zeros((T, wl.n_neurons), np.int64)
    for p, _, k in delivered:
        tot[k, wl.col[p]] += aq[p]
    np.testing.assert_array_equal(r.Iq[:, 0, :].astype(np.int64), tot)


@pytest.mark.parametrize("cap", [1, 2, 4])
def test_drop_rule_replay(cap):
    wl = synth.ragged_network(30, 12, 9, seed=3, rate_hz=600.0, t=300)
    r = oracle.Run(wl, oracle.FIFO, cap, log_events=True)
    S = r.spikes[:, 0, :]
    adm, drp = brute.replay_bounded(S, wl.row_ptr, wl.col, wl.delay_steps, cap)
    dr = r.event_log("dropped")
    assert list(zip(dr["syn"].tolist(), dr["n_emit"].tolist(), dr["k"].tolist())) == drp
    dl = r.event_log("delivered")
    got = set(zip(dl["syn"].tolist(), dl["n_emit"].tolist(), dl["k"].tolist()))
    assert got == {e for e in adm if e[2] < wl.n_steps}
    assert len(drp) > 0
    # sorted kind follows the same rule
    r2 = oracle.Run(wl, oracle.SORTED, cap, log_events=True)
    np.testing.assert_array_equal(r2.spikes, r.spikes)


def test_fifo_capacity_one_is_hold_one_spike():
    wl = synth.ragged_network(25, 8, 6, seed=4, rate_hz=400.0, t=250)
    r = oracle.Run(wl, oracle.FIFO, 1, log_events=True)
    S = r.spikes[:, 0, :]
    want = brute.hold_one_spike(S, wl.row_ptr, wl.col, wl.delay_steps)
    dl = r.event_log("delivered")
    got = set(zip(dl["syn"].tolist(), dl["n_emit"].tolist(), dl["k"].tolist()))
    # the hold model also delivers what is still in flight after the last step: cut at T
    assert got == {e for e in want if e[2] < wl.n_steps}
    assert r.counters()["dropped"] > 0


def _bursty(seed, n=20, fan=6, d_max=9, t=260):
    """A small net whose neurons fire in bursts (strong drive), so that a single synapse often
    holds several events at once."""
    return synth.ragged_network(n, fan, d_max, seed=seed, rate_hz=3000.0, t=t, w_mean=0.3, w_std=0.2)


@pytest.mark.parametrize("cap", [1, 2, 3])
def test_per_synapse_queue_replay(cap):
    """Kind 3 (one bounded FIFO per synapse) against a replay written per synapse from the
    source's spike train alone."""
    wl = _bursty(6)
    r = oracle.Run(wl, oracle.SYN_FIFO, cap, log_events=True)
    S = r.spikes[:, 0, :]
    adm, drp = brute.replay_per_synapse(S, wl.row_ptr, wl.delay_steps, cap)
    dr = r.event_log("dropped")
    assert set(zip(dr["syn"].tolist(), dr["n_emit"].tolist(), dr["k"].tolist())) == drp
    dl = r.event_log("delivered")
    assert set(zip(dl["syn"].tolist(), dl["n_emit"].tolist(), dl["k"].tolist())) == {e for e in adm if e[2] < wl.n_steps}
    c = r.counters()
    assert len(drp) > 50 and c["dropped"] == len(drp) and c["max_occupancy"] == cap
    assert c["enqueued"] == c["delivered"] + c["dropped"] + c["in_flight"]


@pytest.mark.parametrize("cap", [1, 2, 4, 7])
def test_per_synapse_queue_periodic_source_closed_form(cap):
    """A source that fires at every step, through synapses with delays 1..7: the event emitted at
    step n is admitted iff (n mod D) < C when C < D (the queue fills in C steps and a place frees
    every time the oldest event arrives, D steps after it entered), and always when C >= D."""
    n, T = 8, 90
    delays = np.arange(1, 8, dtype=np.uint8)
    row_ptr = np.zeros(n + 1, np.int64); row_ptr[1:] = len(delays)      # all synapses leave neuron 0
    wl = synth.Workload(name="periodic", n_neurons=n, fan_out=len(delays), n_steps=T, batch=1, d_max_steps=7,
                        ext_rate_hz=0.0, seed=1, row_ptr=row_ptr, col=np.arange(1, 8, dtype=np.int32),
                        weight=np.full(len(delays), 0.01, np.float32), delay_steps=delays)
    forced = np.zeros((T, 1, n), np.uint8); forced[:, 0, 0] = 1
    r = oracle.Run(wl, oracle.SYN_FIFO, cap, forced_spikes=forced, log_events=True)
    dr = r.event_log("dropped")
    got = set(zip(dr["syn"].tolist(), dr["n_emit"].tolist()))
    want = {(p, t) for p, d in enumerate(delays.tolist()) for t in range(T) if cap < d and t % d >= cap}
    assert got == want


def test_per_synapse_queue_lossless_equals_ring_and_differs_from_per_target():
    wl = _bursty(9)
    base = oracle.Run(wl, oracle.RING, keep_currents=True)
    occ = oracle.Run(wl, oracle.SYN_FIFO, 10**6).counters()["max_occupancy"]
    assert occ >= 2
    r = oracle.Run(wl, oracle.SYN_FIFO, occ, keep_currents=True)
    np.testing.assert_array_equal(r.U, base.U)
    np.testing.assert_array_equal(r.Iq, base.Iq)
    assert r.counters()["dropped"] == 0
    lossy = oracle.Run(wl, oracle.SYN_FIFO, occ - 1)
    assert lossy.counters()["dropped"] > 0
    # the same capacity per target loses far more: a target's queue is shared by its whole fan-in
    assert oracle.Run(wl, oracle.FIFO, occ - 1).counters()["dropped"] > lossy.counters()["dropped"]


def test_latest_spike_slot_replay():
    """Kind 4 (one slot per synapse, the newest spike replaces the held one) against the rule
    stated from the source's spike train: an event is lost iff its source fires again before it
    arrives."""
    wl = _bursty(12)
    r = oracle.Run(wl, oracle.SYN_LATEST, 1, log_events=True)
    S = r.spikes[:, 0, :]
    kept, lost = brute.replay_latest(S, wl.row_ptr, wl.delay_steps)
    dr = r.event_log("dropped")
    assert set(zip(dr["syn"].tolist(), dr["n_emit"].tolist(), dr["k"].tolist())) == lost
    dl = r.event_log("delivered")
    assert set(zip(dl["syn"].tolist(), dl["n_emit"].tolist(), dl["k"].tolist())) == {e for e in kept if e[2] < wl.n_steps}
    c = r.counters()
    assert len(lost) > 50 and c["dropped"] == len(lost)
    assert c["enqueued"] == c["delivered"] + c["dropped"] + c["in_flight"]
    assert c["sum_enqueued"] == c["sum_delivered"] + c["sum_dropped"] + c["sum_in_flight"]
    # it differs from the slot that keeps the spike it holds (capacity-1 FIFO per synapse)
    assert not np.array_equal(oracle.Run(wl, oracle.SYN_FIFO, 1).U, r.U)


@pytest.mark.parametrize("period", [1, 3, 5, 8])
def test_latest_spike_slot_periodic_source_closed_form(period):
    """A source that fires every `period` steps, synapses with delays 1..7: every event of a synapse
    with delay <= period is delivered, every event of a slower synapse is replaced before it
    arrives (except the last one of the run, which nothing replaces)."""
    n, T = 8, 96
    delays = np.arange(1, 8, dtype=np.uint8)
    row_ptr = np.zeros(n + 1, np.int64); row_ptr[1:] = len(delays)
    wl = synth.Workload(name="periodic", n_neurons=n, fan_out=len(delays), n_steps=T, batch=1, d_max_steps=7,
                        ext_rate_hz=0.0, seed=1, row_ptr=row_ptr, col=np.arange(1, 8, dtype=np.int32),
                        weight=np.full(len(delays), 0.01, np.float32), delay_steps=delays)
    forced = np.zeros((T, 1, n), np.uint8); forced[::period, 0, 0] = 1
    r = oracle.Run(wl, oracle.SYN_LATEST, 1, forced_spikes=forced, log_events=True)
    dr = r.event_log("dropped")
    got = set(zip(dr["syn"].tolist(), dr["n_emit"].tolist()))
    last = (T - 1) // period * period
    want = {(p, t) for p, d in enumerate(delays.tolist()) for t in range(0, T, period) if d > period and t != last}
    assert got == want


@pytest.mark.parametrize("bins", [1, 2, 3, 5])
def test_time_bins_replay(bins):
    """Kind 5 (time bins per synapse, the newer event takes the bin) against a step-by-step replay
    of one ring of spike times per synapse."""
    wl = _bursty(15)
    r = oracle.Run(wl, oracle.SYN_BINS, bins, log_events=True)
    S = r.spikes[:, 0, :]
    kept, lost = brute.replay_time_bins(S, wl.row_ptr, wl.delay_steps, bins)
    dr = r.event_log("dropped")
    assert set(zip(dr["syn"].tolist(), dr["n_emit"].tolist(), dr["k"].tolist())) == lost
    dl = r.event_log("delivered")
    assert set(zip(dl["syn"].tolist(), dl["n_emit"].tolist(), dl["k"].tolist())) == {e for e in kept if e[2] < wl.n_steps}
    c = r.counters()
    assert len(lost) > 20 and c["dropped"] == len(lost)
    assert c["enqueued"] == c["delivered"] + c["dropped"] + c["in_flight"]
    assert c["sum_enqueued"] == c["sum_delivered"] + c["sum_dropped"] + c["sum_in_flight"]


def test_time_bins_special_cases():
    """One bin is the slot that holds the latest spike; as many bins as the largest delay lose
    nothing (the arrivals in flight on a synapse are distinct and less than its delay apart)."""
    wl = _bursty(16)
    one = oracle.Run(wl, oracle.SYN_BINS, 1)
    np.testing.assert_array_equal(one.U, oracle.Run(wl, oracle.SYN_LATEST, 1).U)
    assert one.counters() == oracle.Run(wl, oracle.SYN_LATEST, 1).counters()
    full = oracle.Run(wl, oracle.SYN_BINS, int(wl.delay_steps.max()), keep_currents=True)
    base = oracle.Run(wl, oracle.RING, keep_currents=True)
    np.testing.assert_array_equal(full.U, base.U)
    np.testing.assert_array_equal(full.Iq, base.Iq)
    assert full.counters()["dropped"] == 0
    assert oracle.Run(wl, oracle.SYN_BINS, 2).counters()["dropped"] > 0


@pytest.mark.parametrize("bins,period", [(2, 1), (3, 2), (4, 3), (4, 2), (5, 1)])
def test_time_bins_periodic_source_closed_form(bins, period):
    """A source that fires every `period` steps: the events in flight on a synapse arrive `period`
    apart, so an event is overwritten iff a later one, m periods on, lands in its bin (m * period a
    multiple of `bins`) while it is still in flight (m * period < delay): iff lcm(period, bins) <
    delay -- except the events so late in the run that the overwriting spike never comes."""
    n, T = 8, 120
    delays = np.arange(1, 8, dtype=np.uint8)
    row_ptr = np.zeros(n + 1, np.int64); row_ptr[1:] = len(delays)
    wl = synth.Workload(name="periodic", n_neurons=n, fan_out=len(delays), n_steps=T, batch=1, d_max_steps=7,
                        ext_rate_hz=0.0, seed=1, row_ptr=row_ptr, col=np.arange(1, 8, dtype=np.int32),
                        weight=np.full(len(delays), 0.01, np.float32), delay_steps=delays)
    forced = np.zeros((T, 1, n), np.uint8); forced[::period, 0, 0] = 1
    r = oracle.Run(wl, oracle.SYN_BINS, bins, forced_spikes=forced, log_events=True)
    dr = r.event_log("dropped")
    got = set(zip(dr["syn"].tolist(), dr["n_emit"].tolist()))
    lcm = math.lcm(period, bins)
    want = {(p, t) for p, d in enumerate(delays.tolist()) for t in range(0, T, period)
            if lcm < d and t + lcm < T}
    assert got == want


def test_queue_kinds_agree_when_lossless():
    wl = synth.cfg0(seed=21)
    base = oracle.Run(wl, oracle.RING, keep_currents=True)
    occ = oracle.Run(wl, oracle.FIFO, 10**6).counters()["max_occupancy"]
    for kind in (oracle.FIFO, oracle.SORTED):
        r = oracle.Run(wl, kind, occ, keep_currents=True)
        np.testing.assert_array_equal(r.spikes, base.spikes)
        np.testing.assert_array_equal(r.Iq, base.Iq)
        np.testing.assert_array_equal(r.U, base.U)
        assert r.counters()["dropped"] == 0
    # one slot less must drop something
    assert oracle.Run(wl, oracle.FIFO, occ - 1).counters()["dropped"] > 0


def test_batch_trials_are_independent_and_threading_is_neutral():
    wl = synth.cfg0(seed=8)
    r1 = oracle.Run(wl, oracle.FIFO, 4, batch=3, n_threads=1, n_steps=300)
    r3 = oracle.Run(wl, oracle.FIFO, 4, batch=3, n_threads=3, n_steps=300)
    np.testing.assert_array_equal(r1.U, r3.U)
    assert r1.counters() == r3.counters()
    S = r1.spikes
    assert not np.array_equal(S[:, 0], S[:, 1])   # different drive per trial


def test_erlang_b_sanity_open_loop():
    """A bounded bag with Poisson arrivals and holding time = delay is an
    M/G/c/c loss system; blocking ~ Erlang-B(c, a) (statistical sanity only)."""
    n_src, T, cap = 200, 6000, 4
    rng = np.random.default_rng(0)
    # every source projects once onto target 0 with a random delay
    row_ptr = np.arange(n_src + 2, dtype=np.int64)
    row_ptr[-1] = n_src               # last neuron (the target's own row) is empty
    col = np.full(n_src, n_src, np.int32)
    delay = rng.integers(1, 41, size=n_src).astype(np.uint8)
    wl = synth.Workload("erl", n_src + 1, 1, T, 1, 40, ext_rate_hz=0.0, row_ptr=row_ptr, col=col,
                        weight=np.full(n_src, 1e-4, np.float32), delay_steps=delay)
    p = 0.0007
    forced = np.zeros((T, 1, n_src + 1), np.uint8)
    forced[:, 0, :n_src] = rng.random((T, n_src)) < p
    r = oracle.Run(wl, oracle.FIFO, cap, forced_spikes=forced)
    c = r.counters()
    a = n_src * p * delay.mean()     # offered load = arrival rate x mean holding time
    want = brute.erlang_b(cap, a)
    got = c["dropped"] / c["enqueued"]
    assert 0.02 < want < 0.5
    assert abs(got - want) < 0.25 * want + 0.01


# ---------------------------------------------------------------- continuous delays

def test_continuous_delay_arrival_step_and_amplitude():
    wl = synth.ragged_network(20, 6, 30, seed=9, continuous=True, t=5)
    r = oracle.Run(wl, oracle.RING)
    dt, tau = float(np.float32(wl.dt_ms)), float(np.float32(wl.tau_m_ms))
    d = wl.delay_ms.astype(np.float64)
    D = np.maximum(1, np.ceil(d / dt)).astype(np.int64)
    np.testing.assert_array_equal(r.D, D)
    f = np.exp(-(D * dt - d) / tau)
    np.testing.assert_allclose(r.f_f, f, rtol=1e-7)
    np.testing.assert_allclose(r.a_d, wl.weight.astype(np.float64) * f, rtol=1e-15)
    assert np.all(f <= 1.0) and np.all(f > math.exp(-dt / tau) - 1e-12)
    np.testing.assert_array_equal(r.a_q, np.rint(r.a_d * 2**24).astype(np.int64))


def test_on_grid_continuous_delay_equals_integer_delay():
    wl = synth.cfg0(seed=31)
    a = oracle.Run(wl, oracle.RING)
    wl2 = synth.cfg0(seed=31)
    # a delay exactly representable and exactly on the grid: use dt = 0.125 ms
    wl.dt_ms = wl2.dt_ms = 0.125
    a = oracle.Run(wl, oracle.RING)
    wl2.delay_ms = (wl2.delay_steps.astype(np.float32) * np.float32(0.125))
    wl2.delay_steps = None
    b = oracle.Run(wl2, oracle.RING)
    np.testing.assert_array_equal(a.U, b.U)
    assert np.all(b.f_f == 1.0)


def test_delay_range_errors():
    wl = synth.cfg0()
    wl.delay_steps[3] = 0
    with pytest.raises(oracle.OracleError):
        oracle.Run(wl, oracle.RING)
    wl = synth.cfg0()
    wl.delay_steps[3] = 21
    with pytest.raises(oracle.OracleError):
        oracle.Run(wl, oracle.RING)
