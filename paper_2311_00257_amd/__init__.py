"""MI355X-native model-state step of a ZeRO-style rank on its flat shard of P/G/OS.

``synth`` and ``workloads`` make seeded inputs; ``binding`` is the thin ctypes layer over
the C-ABI library ``libamsp.so`` (hand-written HIP for gfx950).  There is no CPU fallback:
calling a compute entry point without the built library raises.
"""
from . import synth, workloads  # noqa: F401

__all__ = ["synth", "workloads"]
