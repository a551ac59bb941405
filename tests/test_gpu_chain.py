"""The ring's chained step launches (ring_chain.h: the step kernels go to two streams in turn and
wait for one another themselves) against the CPU oracle, through the C ABI: membrane trace bit for
bit, counters, spike counts, both gradients in both gradient modes; block counts from one to the
limit and beyond it (where the launches per step take over), trials, window lengths, runs cut into
pieces and mixed with single steps, resets, rows with more than 64 entries one step away,
continuous delays, agreement with the launches per step, and the failure path of the bounded
waits forced from the host."""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2512_05906_amd import adseq, synth
from tests import helpers as H

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _chain_on(monkeypatch):
    """By default the chained launches run where the resident kernels do not; here wherever the layout allows."""
    monkeypatch.setenv("ADSEQ_RING_CHAIN", "1")


def _run_pieces(wl, T, B, pieces, **kw):
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


@pytest.mark.parametrize("n,fan,b", [(100, 30, 1), (301, 200, 3), (2500, 60, 16), (40000, 20, 1), (131072, 6, 1), (9000, 30, 20)])
def test_chain_forward_sizes(n, fan, b):
    """One block, a few, 157, 512 (the limit) and 704 blocks (beyond it: a launch per step); one trial and many."""
    wl = synth.ragged_network(n, fan, 40, seed=n + b, rate_hz=700.0, t=120, b=b, w_mean=0.6 / fan, w_std=0.4 / fan)
    ref = _check(wl, 120, b, [120])
    assert ref.spikes.sum() > 100


@pytest.mark.parametrize("window", [2, 8, 16, 64])
def test_chain_window_lengths_and_pieces(window, monkeypatch):
    monkeypatch.setenv("ADSEQ_RING_WINDOW", str(window))
    wl = synth.ragged_network(700, 300, 37, seed=5, rate_hz=300.0, t=150, b=2, w_mean=0.004, w_std=0.003)
    ref = _check(wl, 150, 2, [1, 30, "s", "s", 7, 64, "s", 45])
    assert ref.spikes.sum() > 300


def test_chain_matches_step_launches(monkeypatch):
    wl = synth.ragged_network(5000, 80, 50, seed=12, rate_hz=200.0, t=100, b=4, w_mean=0.008, w_std=0.006)
    sim, U1, c1, n1 = _run_pieces(wl, 100, 4, [100])
    sim.close()
    monkeypatch.setenv("ADSEQ_RING_CHAIN", "0")
    monkeypatch.setenv("ADSEQ_RING_RESIDENT", "0")
    sim, U0, c0, n0 = _run_pieces(wl, 100, 4, [100])
    sim.close()
    np.testing.assert_array_equal(U1.view(np.uint32), U0.view(np.uint32))
    assert c1 == c0 and c1["tape_spikes"] > 500
    np.testing.assert_array_equal(n1, n0)


def test_chain_reset_and_rerun():
    wl = synth.ragged_network(1200, 100, 20, seed=3, rate_hz=200.0, t=90, b=2, w_mean=0.006, w_std=0.004)
    sim, U1, c1, _ = _run_pieces(wl, 90, 2, [90])
    sim.reset()
    sim.run(0, 40); sim.run(40, 50)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(sim.tape()["U"].cpu().numpy().view(np.uint32), U1.view(np.uint32))
    assert sim.counters() == c1
    sim.close()


@pytest.mark.parametrize("surrogate", [adseq.SURR_SUPERSPIKE, adseq.GRAD_SPIKE_TIME])
@pytest.mark.parametrize("n,b,T,d_max,continuous", [(700, 3, 150, 40, False), (6000, 2, 100, 40, False),
                                                   (900, 2, 70, 2, False), (1500, 2, 90, 30, True)])
def test_chain_reverse_sweep(surrogate, n, b, T, d_max, continuous, monkeypatch):
    """Both gradients against the oracle, with a cotangent on the membrane values as well, in both
    gradient modes, a run length that is not a multiple of the window; delays of one and two steps
    only (rows of up to 200 entries: more than 64 entries one step away, the gathers beyond a
    wavefront's first load); continuous delays; and agreement with the sweep of one launch per step."""
    wl = synth.ragged_network(n, 200, d_max, seed=n, rate_hz=400.0, t=T, b=b, w_mean=0.004, w_std=0.004,
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
        monkeypatch.setenv("ADSEQ_RING_CHAIN", mode)
        monkeypatch.setenv("ADSEQ_RING_RESIDENT", "0")
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


def test_chain_wait_that_runs_out_is_reported(monkeypatch):
    """Failure path of the bounded waits, forced from the host: with a limit of one poll per wait
    (ADSEQ_RING_RESIDENT_SPINS=1) a launch does not wait for the one before, every kernel still runs
    to its end, the error word carries bit 32, and adseq_drop_count and adseq_backward refuse the
    run; a reset clears the state, and a handle with the ordinary limit gives the oracle's result."""
    wl = synth.ragged_network(40000, 30, 20, seed=21, rate_hz=700.0, t=60, b=2, w_mean=0.02, w_std=0.01)
    monkeypatch.setenv("ADSEQ_RING_RESIDENT_SPINS", "1")
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
    ref = _check(wl, 60, 2, [60])
    assert ref.spikes.sum() > 100
