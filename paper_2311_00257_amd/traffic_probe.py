"""Loader of ``libamsp_probe.so`` (csrc/traffic_probe.hip): traffic-only kernels in the fused step's
access shape.  Used by ``bench.py`` for its ``ceilings``; not part of the product path."""
from __future__ import annotations

import ctypes
import os

from . import build as _build

READ_ONLY, WRITE_ONLY, READ_WRITE = 0, 1, 2

_lib = None


def load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB_PROBE):
            raise RuntimeError("libamsp_probe.so is not built: run `python -m paper_2311_00257_amd.build`")
        import torch  # noqa: F401  (bind to the HIP runtime torch has loaded)

        lib = ctypes.CDLL(_build.LIB_PROBE)
        vp = ctypes.c_void_p
        lib.amsp_probe_traffic.argtypes = [ctypes.c_int, vp, ctypes.c_uint32, vp, vp, vp, vp, ctypes.c_uint64,
                                           ctypes.c_int, vp]
        lib.amsp_probe_traffic.restype = ctypes.c_int
        _lib = lib
    return _lib


def traffic(mode: int, partials, p, m, v, out, n: int, waves_per_cu: int, stream=None) -> None:
    """One launch over the first ``n`` elements (a multiple of 256) of torch device tensors."""
    import torch

    k = len(partials)
    arr = (ctypes.c_void_p * k)(*[t.data_ptr() for t in partials])
    hs = torch.cuda.current_stream().cuda_stream if stream is None else stream
    rc = load().amsp_probe_traffic(mode, arr, k, p.data_ptr(), m.data_ptr(), v.data_ptr(), out.data_ptr(), n,
                                   waves_per_cu, hs or None)
    if rc != 0:
        raise RuntimeError("amsp_probe_traffic failed: %d" % rc)
