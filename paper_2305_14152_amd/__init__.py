"""PEQA quantized-linear hot path for MI355X (gfx950).

`synth` draws seeded synthetic inputs; `peqa` is the thin ctypes binding over the
C-ABI library built from csrc/ (loaded lazily, fails loudly if it is missing).
"""
