"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, sizes workspaces and rejects bad configurations."""
import ctypes as C
import os
import re

import pytest

from paper_2512_05906_amd import adseq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _cfg(**kw):
    base = dict(n_neurons=100, batch=2, d_max_steps=20, capacity=0, kind=adseq.RING, surrogate=0,
                record_tape=1, max_steps=100, dt_ms=0.1, tau_m_ms=20.0, v_thresh=1.0, v_reset=0.0,
                ext_rate_hz=50.0, ext_weight=0.5, seed=1, n_synapses=1000)
    base.update(kw)
    return adseq.Config(**base)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "adseq.h")).read()
    declared = set(re.findall(r"\b(adseq_[a-z_]+)\s*\(", header))
    assert declared == set(adseq.EXPORTS)
    lib = adseq.load()
    for name in declared:
        assert hasattr(lib, name), name


def test_workspace_size_grows_with_the_queue():
    lib = adseq.load()
    ring = lib.adseq_workspace_bytes(C.byref(_cfg()))
    fifo8 = lib.adseq_workspace_bytes(C.byref(_cfg(kind=adseq.FIFO, capacity=8)))
    fifo64 = lib.adseq_workspace_bytes(C.byref(_cfg(kind=adseq.FIFO, capacity=64)))
    assert ring > 0 and fifo8 > 0 and fifo64 > fifo8
    # per slot a 16-bit arrival key and a 32-bit amplitude, one more mask word per target, padding
    assert 56 * 200 * 6 <= fifo64 - fifo8 <= 56 * 200 * 6 + 200 * 4 + 3 * 256
    assert ring % 256 == 0
    # a small ring fits the static workspace of adseq_create_static (its staging for the resident
    # step kernels is sized by the blocks that take part, not by the largest launch)
    assert ring < adseq.STATIC_WORKSPACE_BYTES // 4
    no_tape = lib.adseq_workspace_bytes(C.byref(_cfg(record_tape=0, max_steps=0)))
    assert no_tape < ring
    # one queue per synapse and trial: a 16-bit arrival key per slot
    c2 = _cfg(kind=adseq.SYN_FIFO, capacity=2)
    syn2 = lib.adseq_workspace_bytes(C.byref(c2))
    syn8 = lib.adseq_workspace_bytes(C.byref(_cfg(kind=adseq.SYN_FIFO, capacity=8)))
    queues = c2.batch * c2.n_synapses
    assert abs((syn8 - syn2) - 6 * 2 * queues) <= 256      # up to the 256-byte alignment of the array


@pytest.mark.parametrize("bad", [
    dict(n_neurons=0), dict(batch=0), dict(d_max_steps=0), dict(d_max_steps=1024),
    dict(kind=6), dict(kind=adseq.SYN_LATEST, capacity=2), dict(kind=adseq.SYN_BINS, capacity=9), dict(kind=adseq.SYN_FIFO, capacity=0), dict(kind=adseq.SYN_FIFO, capacity=9),
    dict(kind=adseq.FIFO, capacity=0), dict(kind=adseq.SORTED, capacity=40000),
    dict(dt_ms=0.0), dict(tau_m_ms=0.05), dict(ext_rate_hz=-1.0), dict(n_synapses=-1),
    dict(record_tape=1, max_steps=0), dict(surrogate=5), dict(tau_syn_ms=-1.0), dict(tau_syn_ms=0.05), dict(n_neurons=2**23, d_max_steps=1023),
    dict(tau_rise_ms=0.5), dict(tau_syn_ms=1.0, tau_rise_ms=1.0), dict(tau_syn_ms=1.0, tau_rise_ms=0.05), dict(tau_syn_ms=1.0, tau_rise_ms=-0.5),
])
def test_invalid_configurations_are_rejected_on_the_host(bad):
    lib = adseq.load()
    cfg = _cfg(**bad)
    assert lib.adseq_workspace_bytes(C.byref(cfg)) == 0
    h = C.c_void_p()
    assert lib.adseq_create(C.byref(cfg), C.byref(h)) == -1
    assert not h.value


def test_create_checks_pointers_and_workspace_before_touching_the_gpu():
    lib = adseq.load()
    h = C.c_void_p()
    cfg = _cfg()
    assert lib.adseq_create(C.byref(cfg), C.byref(h)) == -1       # null CSR pointers
    cfg = _cfg(row_ptr=4096, col=4096, weight=4096, delay_steps=4096, delay_ms=4096)
    assert lib.adseq_create(C.byref(cfg), C.byref(h)) == -1       # both delay arrays
    cfg = _cfg(row_ptr=4096, col=4096, weight=4096, delay_steps=4096)
    assert lib.adseq_create(C.byref(cfg), C.byref(h)) == -3       # no workspace
    cfg.workspace, cfg.workspace_bytes = 4096 + 8, 1 << 30
    assert lib.adseq_create(C.byref(cfg), C.byref(h)) == -3       # misaligned
    cfg.workspace, cfg.workspace_bytes = 4096, 1024
    assert lib.adseq_create(C.byref(cfg), C.byref(h)) == -3       # too small
    assert lib.adseq_create(None, C.byref(h)) == -1
    assert not h.value


def test_null_handle_is_an_error_not_a_crash():
    lib = adseq.load()
    assert lib.adseq_destroy(None) == -1
    assert lib.adseq_reset(None, None) == -1
    assert lib.adseq_step(None, 0, None, None, None) == -1
    assert lib.adseq_run(None, 0, 1, None) == -1
    assert lib.adseq_deliver(None, 0, None, None) == -1
    assert lib.adseq_enqueue(None, 0, None, None, None) == -1
    assert lib.adseq_backward(None, None, None, None, None, None) == -1
    assert lib.adseq_drop_count(None, None, None, None, None) == -1
    assert lib.adseq_spike_counts(None, None, None) == -1
    assert lib.adseq_profile(None, 1) == -1
    assert lib.adseq_profile_read(None, None, None, None) == -1
    assert lib.adseq_last_error(None) == b"null handle"
