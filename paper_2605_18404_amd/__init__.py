"""Four-phase (FE / FF / BF / BE) training step of a conservative message-passing
interatomic potential as hand-written HIP kernels for gfx950 behind a C ABI.

`synth` draws the seeded inputs; `binding` is the thin ctypes layer over libmlip.so.
Nothing here computes on the CPU: without the built library the binding raises.
"""
