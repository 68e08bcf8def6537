"""Seeded synthetic model-state inputs (host side).

A stateless, counter-based generator: element ``i`` of tensor ``tensor_id`` under
``seed`` is a pure function of those three integers, so any element of a 100 GB
state can be regenerated on the host without storing it.  Three implementations give the
same bits: the numpy formulas here (``*_at``, any index set), the plain-C contiguous fills
(``csrc/synth_host.c``, used by ``fill_*``) and the device fill kernels
(``csrc/synth_fill.hip``).

Recipe per element:
  1. ``h = splitmix64(key + i * GOLDEN)`` where ``key`` depends on (seed, tensor_id)
     (the published SplitMix64 output function applied to a Weyl sequence);
  2. the top 16 bits of ``h`` index a 65,536-entry fp32 table of standard-normal
     quantiles ``ndtri((j + 0.5) / 65536)``;
  3. one fp32 multiply by the tensor's sigma (and ``fabs`` for the second moment);
  4. for bf16 tensors the low 16 bits of the fp32 pattern are dropped (a mask, not a
     rounding: the generator only has to emit *some* bf16 value of the right scale).

This module holds no arithmetic of the training step itself: it only makes inputs,
for the product, the tests and the CPU oracle alike.  ``i`` is the index in the flat
model-state buffer of the whole model (P/G/OS of Phi elements, Section II-C), so a
shard is a genuine slice of one model.
"""
from __future__ import annotations

import functools

import numpy as np

MASK64 = (1 << 64) - 1
GOLDEN = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB

# tensor ids of the flat model-state streams
TENSOR_MASTER = 0
TENSOR_EXP_AVG = 1
TENSOR_EXP_AVG_SQ = 2
TENSOR_PARTIAL0 = 16  # partial gradient j has id 16 + j


def _mix_int(z: int) -> int:
    z &= MASK64
    z = ((z ^ (z >> 30)) * _M1) & MASK64
    z = ((z ^ (z >> 27)) * _M2) & MASK64
    return z ^ (z >> 31)


def stream_key(seed: int, tensor_id: int) -> int:
    """64-bit key of one tensor's stream."""
    return _mix_int(_mix_int(seed * GOLDEN + 1) ^ ((tensor_id + 1) * _M1))


def _mix_np(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * np.uint64(_M1)
    z = (z ^ (z >> np.uint64(27))) * np.uint64(_M2)
    return z ^ (z >> np.uint64(31))


@functools.lru_cache(maxsize=1)
def normal_table() -> np.ndarray:
    """fp32[65536] standard-normal quantiles at the midpoints of 65,536 equal bins."""
    from scipy.special import ndtri

    q = (np.arange(65536, dtype=np.float64) + 0.5) / 65536.0
    t = ndtri(q).astype(np.float32)
    t.setflags(write=False)
    return t


def table_index_at(key: int, indices: np.ndarray) -> np.ndarray:
    """Table slot (0..65535) for each global element index in ``indices`` (uint64)."""
    idx = np.asarray(indices, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = np.uint64(key) + idx * np.uint64(GOLDEN)
        h = _mix_np(z)
    return (h >> np.uint64(48)).astype(np.int64)


def f32_at(key: int, indices: np.ndarray, sigma: float, absolute: bool = False) -> np.ndarray:
    """fp32 values at arbitrary global indices."""
    z = normal_table()[table_index_at(key, indices)]
    x = z * np.float32(sigma)
    return np.abs(x) if absolute else x


def bf16_at(key: int, indices: np.ndarray, sigma: float) -> np.ndarray:
    """bf16 bit patterns (uint16) at arbitrary global indices."""
    x = f32_at(key, indices, sigma)
    return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


_host_lib = None


def _host():
    """The C implementation of the contiguous fills (csrc/synth_host.c), built on first use."""
    global _host_lib
    if _host_lib is None:
        import ctypes

        from . import build

        lib = ctypes.CDLL(build.build_host_synth())
        u64, vp = ctypes.c_uint64, ctypes.c_void_p
        lib.amsp_synth_host_f32.argtypes = [vp, u64, u64, u64, vp, ctypes.c_float, ctypes.c_int]
        lib.amsp_synth_host_f32.restype = None
        lib.amsp_synth_host_bf16.argtypes = [vp, u64, u64, u64, vp, ctypes.c_float]
        lib.amsp_synth_host_bf16.restype = None
        _host_lib = lib
    return _host_lib


def _parallel(n: int, threads: int, fn) -> None:
    threads = max(1, min(threads, max(1, n // 65536)))
    if threads == 1:
        fn(0, n)
        return
    from concurrent.futures import ThreadPoolExecutor

    edges = [n * c // threads for c in range(threads + 1)]
    with ThreadPoolExecutor(threads) as ex:
        list(ex.map(lambda c: fn(edges[c], edges[c + 1]), range(threads)))


def fill_f32(key: int, index0: int, n: int, sigma: float, absolute: bool = False, out=None,
             threads: int = 1) -> np.ndarray:
    """fp32[n] for global indices index0 .. index0+n-1 (into ``out[:n]`` when given)."""
    out = np.empty(n, dtype=np.float32) if out is None else out[:n]
    assert out.dtype == np.float32 and out.flags.c_contiguous
    lib, table = _host(), normal_table()
    _parallel(n, threads, lambda lo, hi: lib.amsp_synth_host_f32(
        out.ctypes.data + 4 * lo, hi - lo, key, index0 + lo, table.ctypes.data, sigma, int(absolute)))
    return out


def fill_bf16(key: int, index0: int, n: int, sigma: float, out=None, threads: int = 1) -> np.ndarray:
    """bf16[n] (as uint16) for global indices index0 .. index0+n-1 (into ``out[:n]`` when given)."""
    out = np.empty(n, dtype=np.uint16) if out is None else out[:n]
    assert out.dtype == np.uint16 and out.flags.c_contiguous
    lib, table = _host(), normal_table()
    _parallel(n, threads, lambda lo, hi: lib.amsp_synth_host_bf16(
        out.ctypes.data + 2 * lo, hi - lo, key, index0 + lo, table.ctypes.data, sigma))
    return out


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to fp32 (exact; a view, no rounding)."""
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)
