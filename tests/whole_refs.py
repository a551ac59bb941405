"""Oracle runs of the large configurations at their own length, for tests/test_gpu_whole_configs.py.

One oracle run of the headline network over its 1,000 steps takes minutes on one core (2e8 events
through one priority queue), so all the long runs are started in background threads when the test
session has collected that module (tests/conftest.py) and overlap with each other and with the
GPU tests that come before; a test takes its reference with get(name), which waits for the run.
Every run appends a line per 50 time steps of its first trial, and one per further trial, to
the progress log in the run's output folder (the oracle's own progress hook), so that a long wait is not
mistaken for a hang.  The four runs of config 4 (256 trials over 5,000 steps: 47 GB inside the
oracle each) take turns in one worker of their own, with 16 threads over the trials."""
import os
import threading
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from oracle import oracle
from paper_2512_05906_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

_lock = threading.Lock()
_workloads = {}
_pool = None
_pool_batched = None
_futures = {}

# name -> (workload key, oracle kind, capacity, steps, gradients wanted)
JOBS = {
    "cfg3_ring_T1000": ("cfg3", oracle.RING, 0, 1000, True),
    "cfg3_fifo32_T1000": ("cfg3", oracle.FIFO, 32, 1000, True),
    "cfg3_synfifo4_T1000": ("cfg3", oracle.SYN_FIFO, 4, 1000, True),
    "cfg3_sorted32_T1000": ("cfg3", oracle.SORTED, 32, 1000, True),
    "cfg3_latest_T1000": ("cfg3", oracle.SYN_LATEST, 1, 1000, True),
    "cfg3_bins4_T1000": ("cfg3", oracle.SYN_BINS, 4, 1000, True),
    "cfg3_sorted32_T300": ("cfg3_55hz", oracle.SORTED, 32, 300, True),
    "cfg3_latest_T300": ("cfg3_55hz", oracle.SYN_LATEST, 1, 300, True),
    "cfg2_ring_T10000": ("cfg2_5hz", oracle.RING, 0, 10000, False),
    "cfg2_fifo8_T10000": ("cfg2_5hz", oracle.FIFO, 8, 10000, False),
    "cfg2_fifo32_T10000": ("cfg2_5hz", oracle.FIFO, 32, 10000, False),
    "cfg2_20hz_ring_T10000": ("cfg2_20hz", oracle.RING, 0, 10000, False),
    "cfg2_20hz_fifo8_T10000": ("cfg2_20hz", oracle.FIFO, 8, 10000, False),
    "cfg2_20hz_fifo32_T10000": ("cfg2_20hz", oracle.FIFO, 32, 10000, False),
    "cfg2_20hz_synfifo4_T10000": ("cfg2_20hz", oracle.SYN_FIFO, 4, 10000, False),
    "cfg4_sorted128_T5000": ("cfg4", oracle.SORTED, 128, 5000, True),
    "cfg4_fifo32_T5000": ("cfg4", oracle.FIFO, 32, 5000, True),
    "cfg4_ring_T5000": ("cfg4", oracle.RING, 0, 5000, True),
    "cfg4_synfifo4_T5000": ("cfg4", oracle.SYN_FIFO, 4, 5000, True),
}


def workload(key):
    with _lock:
        if key not in _workloads:
            if key == "cfg3":            # the run bench.py times: drive tuned for a 20 Hz run average
                _workloads[key] = synth.cfg3()
            elif key == "cfg3_55hz":     # a stronger drive, so that 300 steps already carry 2.5e7 events
                _workloads[key] = synth.cfg3(rate_hz=55.0, n_steps=300)
            elif key == "cfg2_5hz":      # config 2 with the drive tuned for 5 Hz
                _workloads[key] = synth.cfg2(rate_hz=synth.CFG2_DRIVE_HZ[5])
            elif key == "cfg2_20hz":     # ... and for 20 Hz
                _workloads[key] = synth.cfg2(rate_hz=synth.CFG2_DRIVE_HZ[20])
            elif key == "cfg4":          # config 4 as it is written: 256 trials, 5,000 steps, 10 Hz drive
                _workloads[key] = synth.cfg4()
            else:
                raise KeyError(key)
        return _workloads[key]


def dL_dcount(wl, counts):
    """Cotangent of the mean squared error between spike counts and the seeded targets."""
    y = synth.spike_count_targets(wl)
    return (2.0 * (counts.astype(np.float32) - y) / np.float32(wl.batch * wl.n_neurons)).astype(np.float32)


def _job(name):
    key, kind, cap, T, grads = JOBS[name]
    wl = workload(key)
    ref = oracle.Run(wl, kind, cap, n_steps=T, n_threads=16 if wl.batch > 1 else 1)
    out = dict(U=ref.U, counters=ref.counters())
    counts = np.zeros((wl.batch, wl.n_neurons), dtype=np.int64)
    spikes = ref.spikes
    for n0 in range(0, T, 256):     # (in slices: the sum of a 5 GB raster would widen it to 8 bytes per entry)
        counts += spikes[n0:n0 + 256].sum(axis=0, dtype=np.int64)
    del spikes
    out["counts"] = counts.astype(np.int32)
    if grads:
        out["dL_dc"] = dL_dcount(wl, counts)
        out["gw"], out["gd"] = ref.backward(out["dL_dc"], None)
    ref.close()
    return out


def start(names=None):
    """Starts the oracle runs in background threads (once)."""
    global _pool, _pool_batched
    with _lock:
        if _pool is not None:
            return
        os.makedirs(os.path.join(ROOT, "gpurun_out"), exist_ok=True)
        os.environ.setdefault("ORACLE_PROGRESS_FILE", os.path.join(ROOT, "gpurun_out", "oracle_progress.log"))
        _pool = ThreadPoolExecutor(max_workers=len(JOBS))
        _pool_batched = ThreadPoolExecutor(max_workers=1)
    for name in (names or JOBS):
        pool = _pool_batched if workload_batch(name) > 1 else _pool
        _futures[name] = pool.submit(_job, name)


def workload_batch(name):
    return 256 if JOBS[name][0] == "cfg4" else 1


def get(name):
    """The reference of one run (waits for it; starts it if nothing was started ahead)."""
    if name not in _futures:
        start([name])
    return _futures[name].result()


def drop(name):
    """Lets go of a reference that has been used (the large ones are tens of GB)."""
    _futures.pop(name, None)
