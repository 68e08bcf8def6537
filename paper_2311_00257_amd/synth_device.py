"""Device side of the seeded input generator: fills torch device tensors with the bits
``synth`` produces on the host, through ``libamsp_synth.so`` (csrc/synth_fill.hip)."""
from __future__ import annotations

import ctypes
import os

from . import build as _build
from . import synth

_lib = None
_tables = {}


def load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB_SYNTH):
            raise RuntimeError("libamsp_synth.so is not built: run `python -m paper_2311_00257_amd.build`")
        # torch supplies the device memory these kernels touch, so the library must bind to the
        # HIP runtime torch has loaded: importing torch first makes the dynamic linker reuse it
        # (two HIP runtimes in one process do not see each other's device state).
        import torch  # noqa: F401

        lib = ctypes.CDLL(_build.LIB_SYNTH)
        u64, vp = ctypes.c_uint64, ctypes.c_void_p
        lib.amsp_synth_fill_f32.argtypes = [vp, u64, u64, u64, vp, ctypes.c_float, ctypes.c_int, vp]
        lib.amsp_synth_fill_f32.restype = ctypes.c_int
        lib.amsp_synth_fill_bf16.argtypes = [vp, u64, u64, u64, vp, ctypes.c_float, vp]
        lib.amsp_synth_fill_bf16.restype = ctypes.c_int
        _lib = lib
    return _lib


def _table(device):
    import torch

    key = str(device)
    if key not in _tables:
        _tables[key] = torch.from_numpy(synth.normal_table().copy()).to(device)
    return _tables[key]


def _stream():
    import torch

    return torch.cuda.current_stream().cuda_stream or None


def fill_f32(out, key: int, index0: int, sigma: float, absolute: bool = False) -> None:
    """out: contiguous float32 device tensor; element i gets the value of global index index0 + i."""
    import torch

    assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous()
    rc = load().amsp_synth_fill_f32(out.data_ptr(), out.numel(), key, index0, _table(out.device).data_ptr(),
                                    sigma, int(absolute), _stream())
    if rc != 0:
        raise RuntimeError("amsp_synth_fill_f32 failed")


def fill_bf16(out, key: int, index0: int, sigma: float) -> None:
    """out: contiguous 2-byte device tensor (bfloat16 / int16 / uint16) receiving bf16 patterns."""
    assert out.is_cuda and out.element_size() == 2 and out.is_contiguous()
    rc = load().amsp_synth_fill_bf16(out.data_ptr(), out.numel(), key, index0, _table(out.device).data_ptr(),
                                     sigma, _stream())
    if rc != 0:
        raise RuntimeError("amsp_synth_fill_bf16 failed")
