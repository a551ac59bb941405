"""adseq_create_static (the entry point that allocates nothing: its workspace is a static array
inside the library's device image) against adseq_create with a caller-provided workspace, through
the C ABI: two calls in a row on the shared static workspace, the second with a smaller network.
Membrane trace, raster, counters and spike counts bit for bit; gradients to the tolerance of the
parity tests (fp32 atomic order differs between runs)."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2512_05906_amd import adseq, synth
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _run(wl, kind, cap, T, B, static):
    sim = adseq.Adseq(wl, kind, cap, batch=B, record_tape=True, max_steps=T, static_workspace=static)
    assert sim.workspace_bytes <= adseq.STATIC_WORKSPACE_BYTES
    S = torch.zeros((T, B, wl.n_neurons), dtype=torch.uint8, device=sim.dev)
    for n in range(T):
        sim.step(n, None, S[n])
    torch.cuda.synchronize()
    out = dict(S=S.cpu().numpy(), U=sim.tape()["U"].cpu().numpy().copy(), counters=sim.counters())
    counts = torch.empty(B * wl.n_neurons, dtype=torch.int32, device=sim.dev)
    sim.spike_counts(counts)
    out["counts"] = counts.cpu().numpy()
    rng = np.random.default_rng(5)
    dc = torch.from_numpy(rng.normal(0, 1e-3, (B, wl.n_neurons)).astype(np.float32)).to(sim.dev)
    g_w = torch.empty(wl.n_synapses, device=sim.dev)
    g_d = torch.empty(wl.n_synapses, device=sim.dev)
    sim.backward(dc, None, g_w, g_d)
    torch.cuda.synchronize()
    out["gw"], out["gd"] = g_w.cpu().numpy(), g_d.cpu().numpy()
    sim.close()
    return out


def _same(a, b):
    np.testing.assert_array_equal(a["S"], b["S"])
    np.testing.assert_array_equal(a["U"].view(np.uint32), b["U"].view(np.uint32))
    np.testing.assert_array_equal(a["counts"], b["counts"])
    assert a["counters"] == b["counters"] and a["counters"]["error_bits"] == 0
    assert a["S"].sum() > 50
    H.grad_close(a["gw"], b["gw"])
    H.grad_close(a["gd"], b["gd"])
    assert np.abs(b["gw"]).max() > 0


@pytest.mark.parametrize("kind,cap", [(adseq.RING, 0), (adseq.FIFO, 3)])
def test_static_workspace_matches_caller_workspace(kind, cap):
    big = synth.ragged_network(300, 400, 30, seed=3, rate_hz=200.0, t=150, b=2, w_mean=0.01, w_std=0.01)
    small = synth.ragged_network(90, 120, 12, seed=4, rate_hz=250.0, t=80, b=1, w_mean=0.02, w_std=0.01)
    for wl, T, B in ((big, 150, 2), (small, 80, 1)):   # the second call reuses the workspace the first left behind
        _same(_run(wl, kind, cap, T, B, static=True), _run(wl, kind, cap, T, B, static=False))


def test_static_workspace_limits():
    lib = adseq.load()
    wl = synth.ragged_network(90, 120, 12, seed=4, rate_hz=250.0, t=80, b=1, w_mean=0.02, w_std=0.01)
    # a tape that does not fit the static workspace is refused
    with pytest.raises(adseq.AdseqError) as e:
        adseq.Adseq(wl, adseq.RING, 0, record_tape=True, max_steps=200000, static_workspace=True)
    assert e.value.code == -3
    # one live handle per device; destroying it frees the workspace again
    a = adseq.Adseq(wl, adseq.RING, 0, static_workspace=True)
    with pytest.raises(adseq.AdseqError) as e:
        adseq.Adseq(wl, adseq.RING, 0, static_workspace=True)
    assert e.value.code == -3
    a.close()
    b = adseq.Adseq(wl, adseq.RING, 0, static_workspace=True)
    b.run(0, 10)
    torch.cuda.synchronize()
    assert b.counters()["error_bits"] == 0
    b.close()
    assert lib.adseq_create_static(None, None) == -1
