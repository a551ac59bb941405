"""Open-loop queues fed by Poisson sources (the shape of the paper's Poisson benchmark,
Section 5.1: independent queues, one source each, one homogeneous delay): HIP path vs oracle
bit for bit, and the drop rate against the Erlang-B blocking probability."""
import numpy as np
import pytest
import torch

from oracle import brute, oracle
from paper_2512_05906_amd import adseq, synth

pytestmark = pytest.mark.gpu

KINDS = {"ring": oracle.RING, "fifo": oracle.FIFO, "sorted": oracle.SORTED, "syn": oracle.SYN_FIFO, "latest": oracle.SYN_LATEST, "bins": oracle.SYN_BINS}


@pytest.mark.parametrize("kind,cap,interval", [("ring", 0, 400), ("fifo", 1, 400), ("fifo", 2, 80),
                                               ("fifo", 4, 40), ("sorted", 4, 40), ("fifo", 40, 40), ("syn", 4, 40),
                                               ("syn", 1, 400), ("latest", 1, 40), ("bins", 4, 40)])
def test_poisson_queues_open_loop(kind, cap, interval):
    N, T, delay = 1500, 3000, 80          # 1,500 queues: several blocks and a ragged tail
    wl = synth.poisson_queues(N, delay, n_steps=T)
    rate_hz = 1.0 / (interval * wl.dt_ms * 1e-3)
    lists = synth.poisson_spike_lists(N, 1, T, rate_hz, wl.dt_ms, seed=5)
    forced = np.zeros((T, N), np.uint8)
    for n, ids in enumerate(lists):
        forced[n, ids] = 1
    ref = oracle.Run(wl, KINDS[kind], cap, n_steps=T, forced_spikes=forced.reshape(T, 1, N), keep_currents=True)
    sim = adseq.Adseq(wl, KINDS[kind], cap)
    I = torch.zeros((T, N), dtype=torch.float32, device=sim.dev)
    counts = torch.tensor([len(x) for x in lists], dtype=torch.int32, device=sim.dev)
    offs = np.concatenate([[0], np.cumsum([len(x) for x in lists])])
    ids = torch.from_numpy(np.concatenate(lists + [np.zeros(1, np.int32)])).to(sim.dev)
    # first third through the batched entry point, second step by step, the rest batched again
    # (for the ring the batched entry point pops and enqueues a step in one launch: both hand-overs)
    a, b = T // 3, 2 * T // 3
    sim.run_open(0, a, ids, offs[:a], counts, I, N)
    for n in range(a, b):
        sim.deliver(n, I[n])
        sim.enqueue(n, ids[int(offs[n]):], counts[n:])
    sim.run_open(b, T - b, ids, offs[b:T], counts[b:], I[b:], N)
    torch.cuda.synchronize()
    want = ref.Iq.reshape(T, N).astype(np.float32) * np.float32(2.0 ** -24)
    np.testing.assert_array_equal(I.cpu().numpy().view(np.uint32), want.view(np.uint32))
    c, rc = sim.counters(), ref.counters()
    for key in ("enqueued", "dropped", "delivered", "sum_enqueued", "sum_dropped", "sum_delivered"):
        assert c[key] == rc[key], key
    sim.close()
    if kind == "ring" or cap >= 40:
        assert rc["dropped"] == 0
    elif kind == "bins":
        # an event is lost iff its source fires again a multiple of `cap` steps later, before it
        # arrives: at one of the (delay - 1) // cap such steps
        want_p = 1.0 - (1.0 - 1.0 / interval) ** ((delay - 1) // cap)
        got = rc["dropped"] / rc["enqueued"]
        assert abs(got - want_p) < 0.03, (got, want_p)
    elif kind == "latest":
        # an event is lost iff its source fires again in one of the delay - 1 steps before it arrives
        want_p = 1.0 - (1.0 - 1.0 / interval) ** (delay - 1)
        got = rc["dropped"] / rc["enqueued"]
        assert abs(got - want_p) < 0.03, (got, want_p)
    else:
        # loss system with `cap` servers, offered load = delay / mean interval
        want_b = brute.erlang_b(cap, delay / interval)
        got = rc["dropped"] / rc["enqueued"]
        assert abs(got - want_b) < 0.1 * want_b + 0.01, (got, want_b)
