"""MI355X-native entropy-coding stage of PILC (arXiv 2206.05279).

`binding` holds the thin ctypes layer over the C-ABI library (libpilc.so, built
from csrc/ with hipcc for gfx950); `synth` holds the seeded workload generators.
Nothing here falls back to a CPU implementation: without the built library the
binding raises.
"""
__all__ = ["binding", "synth"]
