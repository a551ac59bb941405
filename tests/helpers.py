"""Shared helpers of the GPU parity tests: run the HIP path through the C ABI
and collect what is compared with the oracle."""
import numpy as np
import torch

from paper_2512_05906_amd import adseq


def run_gpu(wl, kind, capacity=0, *, n_steps=None, batch=None, record=True, i_ext=None,
            per_step=True, surrogate=0, **kw):
    """Runs T closed-loop steps; returns the handle and a dict of host arrays."""
    T = wl.n_steps if n_steps is None else n_steps
    B = wl.batch if batch is None else batch
    sim = adseq.Adseq(wl, kind, capacity, batch=B, record_tape=record, max_steps=T,
                      surrogate=surrogate, **kw)
    out = {}
    if per_step:
        S = torch.zeros((T, B, wl.n_neurons), dtype=torch.uint8, device=sim.dev)
        ext = None if i_ext is None else torch.from_numpy(np.ascontiguousarray(i_ext, np.float32)).to(sim.dev)
        for n in range(T):
            sim.step(n, None if ext is None else ext[n], S[n])
        out["S"] = S.cpu().numpy()
    else:
        sim.run(0, T)
    torch.cuda.synchronize()
    out["counters"] = sim.counters()
    if record:
        tp = sim.tape()
        out["U"] = tp["U"].cpu().numpy()
        if "step_offset" in tp:
            out["step_offset"] = tp["step_offset"].cpu().numpy()
            out["spike_id"] = tp["spike_id"].cpu().numpy()
        if "event_base" in tp:
            out["event_base"] = tp["event_base"].cpu().numpy()
    return sim, out


def gpu_dropped_set(sim, out, wl):
    """{(syn, n_emit, b)} of events refused by a full queue, from the admission flags."""
    off, ids, evb = out["step_offset"], out["spike_id"], out["event_base"]
    dropped, admitted = set(), set()
    N = wl.n_neurons
    for n in range(len(off) - 1):
        for e in range(off[n], off[n + 1]):
            g = int(ids[e]); b, i = divmod(g, N)
            r0, r1 = int(wl.row_ptr[i]), int(wl.row_ptr[i + 1])
            if r1 == r0:
                continue
            fl = sim.admitted_flags(int(evb[e]), r1 - r0).cpu().numpy()
            for q in range(r1 - r0):
                (admitted if fl[q] else dropped).add((r0 + q, n, b))
    return admitted, dropped


def oracle_sets(r):
    dl, dr = r.event_log("delivered"), r.event_log("dropped")
    delivered = set(zip(dl["syn"].tolist(), dl["n_emit"].tolist(), dl["b"].tolist()))
    dropped = set(zip(dr["syn"].tolist(), dr["n_emit"].tolist(), dr["b"].tolist()))
    return delivered, dropped


def spikes_from_tape(out, wl, B):
    """Raster [T,B,N] rebuilt from the recorded spike lists."""
    off, ids = out["step_offset"], out["spike_id"]
    T = len(off) - 1
    S = np.zeros((T, B * wl.n_neurons), np.uint8)
    for n in range(T):
        S[n, ids[off[n]:off[n + 1]]] = 1
    return S.reshape(T, B, wl.n_neurons)


def grad_close(got, want, rtol=1e-5, atol=1e-6, l2=1e-5):
    """Element-wise 1e-5 relative / 1e-6 absolute and relative L2 <= 1e-5."""
    got = np.asarray(got, np.float64); want = np.asarray(want, np.float64)
    np.testing.assert_allclose(got, want, rtol=rtol, atol=atol)
    den = np.linalg.norm(want)
    if den > 0:
        assert np.linalg.norm(got - want) / den <= l2, np.linalg.norm(got - want) / den
