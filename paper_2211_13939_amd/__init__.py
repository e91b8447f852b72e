"""Pooled incremental Tacotron-2-style decoder step for MI355X (gfx950).

`synth` draws the seeded synthetic inputs; `binding` is the thin ctypes layer
over the C-ABI library built from `csrc/` (loaded lazily, so that CPU-only
tools can import this package without a GPU).
"""
