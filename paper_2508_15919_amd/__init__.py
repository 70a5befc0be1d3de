"""libhfxattn: mixed prefill/decode paged attention for one scheduled serving step on MI355X.

`synth` makes seeded inputs (numpy only).  `binding` is the thin ctypes layer over the
C-ABI library built from `csrc/`; it is imported on first use so that input generation
works without the GPU library, while every compute call fails loudly if it is missing.
"""

__all__ = ["synth", "binding", "build"]
