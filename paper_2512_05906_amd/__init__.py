"""MI355X-native delayed spike-event delivery (ADSEQ hot path).

`synth` draws the seeded synthetic networks; `adseq` is the thin binding over
the C-ABI HIP library (loaded on first use; it raises if the library is missing).
"""
