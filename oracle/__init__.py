"""Python face of the CPU oracle (``amsp_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by the tests, by the smoke check and by the
benchmark's CPU-baseline leg, never by the product package.  The arithmetic lives in
the C file; this module compiles it with gcc, marshals numpy arrays and, when asked for
more than one thread, hands each thread one contiguous chunk (the per-chunk squared
norms are then added in chunk order).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "amsp_oracle.c")
_LIB = os.path.join(_HERE, "libamsp_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 (no fast-math) into ``libamsp_oracle.so``.  With AMSP_ORACLE_UBSAN=1
    in the environment (the sanitizer tier of the tests sets it for a run of the pins) a second library,
    instrumented with -fsanitize=undefined and aborting on the first report, is built and used instead."""
    ubsan = os.environ.get("AMSP_ORACLE_UBSAN") == "1"
    lib = _LIB.replace(".so", "_ubsan.so") if ubsan else _LIB
    if force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(_SRC):
        tmp = lib + ".tmp%d" % os.getpid()
        flags = ["-O1", "-g", "-fsanitize=undefined", "-fno-sanitize-recover=all"] if ubsan else ["-O2"]
        subprocess.check_call(["gcc", *flags, "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, lib)
    return lib


def _bind(lib):
    """Declare the C signatures on a loaded library (also used by the tests that load
    deliberately broken builds of the oracle to show that the pins catch them)."""
    u64, u32, dbl, flt, vp = ctypes.c_uint64, ctypes.c_uint32, ctypes.c_double, ctypes.c_float, ctypes.c_void_p
    lib.amsp_oracle_shard_range.argtypes = [u64, u32, u32, ctypes.POINTER(u64), ctypes.POINTER(u64)]
    lib.amsp_oracle_shard_range.restype = None
    lib.amsp_oracle_reduce.argtypes = [vp, u32, u64, vp]
    lib.amsp_oracle_reduce.restype = None
    lib.amsp_oracle_sqnorm.argtypes = [vp, u64]
    lib.amsp_oracle_sqnorm.restype = dbl
    lib.amsp_oracle_clip_scale.argtypes = [dbl, dbl, dbl]
    lib.amsp_oracle_clip_scale.restype = dbl
    lib.amsp_oracle_adamw.argtypes = [vp, dbl, vp, vp, vp, u64, flt, flt, flt, flt, flt, u32, vp, vp, vp]
    lib.amsp_oracle_adamw.restype = None
    lib.amsp_oracle_bf16_rne.argtypes = [flt]
    lib.amsp_oracle_bf16_rne.restype = ctypes.c_uint16
    lib.amsp_oracle_cast.argtypes = [vp, u64, vp]
    lib.amsp_oracle_cast.restype = None
    lib.amsp_oracle_round_f32.argtypes = [vp, u64, vp]
    lib.amsp_oracle_round_f32.restype = None
    lib.amsp_oracle_e4m3_decode.argtypes = [ctypes.c_uint8]
    lib.amsp_oracle_e4m3_decode.restype = flt
    lib.amsp_oracle_e4m3_encode.argtypes = [flt]
    lib.amsp_oracle_e4m3_encode.restype = ctypes.c_uint8
    lib.amsp_oracle_absmax.argtypes = [vp, u64]
    lib.amsp_oracle_absmax.restype = flt
    lib.amsp_oracle_fp8_scale.argtypes = [flt]
    lib.amsp_oracle_fp8_scale.restype = flt
    lib.amsp_oracle_cast_fp8.argtypes = [vp, u64, flt, vp]
    lib.amsp_oracle_cast_fp8.restype = None
    return lib


def _load():
    global _lib
    if _lib is None:
        _lib = _bind(ctypes.CDLL(build()))
    return _lib


def _ptr(a: np.ndarray) -> int:
    return a.ctypes.data


def _chunks(n: int, threads: int):
    threads = max(1, min(threads, n if n > 0 else 1))
    edges = [n * c // threads for c in range(threads + 1)]
    return [(edges[c], edges[c + 1]) for c in range(threads) if edges[c + 1] > edges[c]]


def _run(fn, n: int, threads: int):
    parts = _chunks(n, threads)
    if len(parts) <= 1:
        return [fn(lo, hi) for lo, hi in parts]
    with ThreadPoolExecutor(len(parts)) as ex:
        return list(ex.map(lambda c: fn(*c), parts))


def shard_range(total: int, shard_factor: int, rank: int):
    b, e = ctypes.c_uint64(), ctypes.c_uint64()
    _load().amsp_oracle_shard_range(total, shard_factor, rank, ctypes.byref(b), ctypes.byref(e))
    return b.value, e.value


def reduce(partials, threads: int = 1) -> np.ndarray:
    """partials: sequence of k uint16 (bf16 bit pattern) arrays of equal length -> float64 sum."""
    lib = _load()
    parts = [np.ascontiguousarray(p, dtype=np.uint16) for p in partials]
    k, n = len(parts), (parts[0].size if parts else 0)
    assert all(p.size == n for p in parts)
    G = np.empty(n, dtype=np.float64)

    def work(lo, hi):
        ptrs = (ctypes.c_void_p * k)(*[_ptr(p) + 2 * lo for p in parts])
        lib.amsp_oracle_reduce(ctypes.cast(ptrs, ctypes.c_void_p), k, hi - lo, _ptr(G) + 8 * lo)

    _run(work, n, threads)
    return G


def sqnorm(G: np.ndarray, threads: int = 1) -> float:
    lib = _load()
    G = np.ascontiguousarray(G, dtype=np.float64)
    parts = _run(lambda lo, hi: lib.amsp_oracle_sqnorm(_ptr(G) + 8 * lo, hi - lo), G.size, threads)
    total = 0.0
    for s in parts:
        total += s
    return total


def clip_scale(total_sqnorm: float, max_norm: float, clip_eps: float = 1e-6) -> float:
    return _load().amsp_oracle_clip_scale(float(total_sqnorm), float(np.float32(max_norm)),
                                          float(np.float32(clip_eps)))


def adamw(G, scale, p, m, v, *, lr, beta1, beta2, eps, weight_decay, step, threads: int = 1):
    """One AdamW step in double from fp32 state; returns (p', m', v') as float64 arrays."""
    lib = _load()
    G = np.ascontiguousarray(G, dtype=np.float64)
    p = np.ascontiguousarray(p, dtype=np.float32)
    m = np.ascontiguousarray(m, dtype=np.float32)
    v = np.ascontiguousarray(v, dtype=np.float32)
    n = G.size
    assert p.size == n and m.size == n and v.size == n
    po, mo, vo = (np.empty(n, dtype=np.float64) for _ in range(3))

    def work(lo, hi):
        lib.amsp_oracle_adamw(_ptr(G) + 8 * lo, float(scale), _ptr(p) + 4 * lo, _ptr(m) + 4 * lo,
                              _ptr(v) + 4 * lo, hi - lo, lr, beta1, beta2, eps, weight_decay, int(step),
                              _ptr(po) + 8 * lo, _ptr(mo) + 8 * lo, _ptr(vo) + 8 * lo)

    _run(work, n, threads)
    return po, mo, vo


def bf16_rne(x: float) -> int:
    return int(_load().amsp_oracle_bf16_rne(float(np.float32(x))))


def cast(p: np.ndarray, threads: int = 1) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest even."""
    lib = _load()
    p = np.ascontiguousarray(p, dtype=np.float32)
    out = np.empty(p.size, dtype=np.uint16)
    _run(lambda lo, hi: lib.amsp_oracle_cast(_ptr(p) + 4 * lo, hi - lo, _ptr(out) + 2 * lo), p.size, threads)
    return out


def round_f32(x: np.ndarray) -> np.ndarray:
    """double -> fp32, round to nearest even (the C conversion)."""
    lib = _load()
    x = np.ascontiguousarray(x, dtype=np.float64)
    out = np.empty(x.size, dtype=np.float32)
    lib.amsp_oracle_round_f32(_ptr(x), x.size, _ptr(out))
    return out


def step(partials, p, m, v, *, lr, beta1, beta2, eps, weight_decay, step, max_norm, clip_eps=1e-6,
         other_ranks_sqnorm: float = 0.0, threads: int = 1):
    """The whole path on one shard: reduce -> squared norm -> clip scale -> AdamW -> cast.

    Returns a dict with G (float64), sqnorm, scale, p/m/v (float64), p_f32/m_f32/v_f32
    (rounded) and p_bf16 (bit patterns of bf16(fp32(p')))."""
    G = reduce(partials, threads)
    S = sqnorm(G, threads)
    scale = clip_scale(S + other_ranks_sqnorm, max_norm, clip_eps)
    p1, m1, v1 = adamw(G, scale, p, m, v, lr=lr, beta1=beta1, beta2=beta2, eps=eps,
                       weight_decay=weight_decay, step=step, threads=threads)
    p32 = round_f32(p1)
    return dict(G=G, sqnorm=S, scale=scale, p=p1, m=m1, v=v1, p_f32=p32, m_f32=round_f32(m1),
                v_f32=round_f32(v1), p_bf16=cast(p32, threads))


# --------------------------------------------------------------------------- inter-tensor shards
# Section IV-C.2, second scheme: every parameter tensor goes, whole, with its optimizer states,
# to one rank, "using a greedy algorithm to balance GPU memory usage"; after the gradient
# AllReduce a rank keeps ("selects") the gradients of the tensors it owns and drops the rest.
# The paper does not spell the greedy rule out; the reading taken here: tensors are visited in
# model order and each goes to the rank that holds the fewest elements so far, the lowest such
# rank on a tie.

def partition_tensors(sizes, shard_factor: int):
    """owner[i] for every tensor, by the greedy rule above.  Pure integers."""
    load = [0] * shard_factor
    owner = []
    for sz in sizes:
        r = min(range(shard_factor), key=lambda q: (load[q], q))
        owner.append(r)
        load[r] += int(sz)
    return owner


def owned_segments(sizes, owner, rank: int):
    """Rank's shard as a list of (flat_offset, local_offset, length): its tensors in model order,
    neighbours in the flat buffer merged, stored back to back in the rank's compact OS buffers.
    Empty tensors contribute nothing."""
    segs = []
    flat = 0
    local = 0
    for sz, o in zip(sizes, owner):
        sz = int(sz)
        if o == rank and sz > 0:
            if segs and segs[-1][0] + segs[-1][2] == flat:
                segs[-1] = (segs[-1][0], segs[-1][1], segs[-1][2] + sz)
            else:
                segs.append((flat, local, sz))
            local += sz
        flat += sz
    return segs


def select(flat_array: np.ndarray, segments) -> np.ndarray:
    """The owned elements of a flat (whole-model) array, in compact order: "select & drop"."""
    if not segments:
        return flat_array[:0].copy()
    return np.concatenate([flat_array[f:f + n] for f, _, n in segments])


# --------------------------------------------------------------------------- FP8 payload
def e4m3_decode(code: int) -> float:
    return float(_load().amsp_oracle_e4m3_decode(int(code)))


def e4m3_encode(x: float) -> int:
    return int(_load().amsp_oracle_e4m3_encode(float(np.float32(x))))


def absmax(p: np.ndarray) -> float:
    p = np.ascontiguousarray(p, dtype=np.float32)
    return float(_load().amsp_oracle_absmax(_ptr(p), p.size))


def fp8_scale(amax: float) -> float:
    return float(_load().amsp_oracle_fp8_scale(float(np.float32(amax))))


def cast_fp8(p: np.ndarray, scale: float) -> np.ndarray:
    """e4m3 codes (uint8) of p * scale, the product and the scale in fp32."""
    p = np.ascontiguousarray(p, dtype=np.float32)
    out = np.empty(p.size, dtype=np.uint8)
    _load().amsp_oracle_cast_fp8(_ptr(p), p.size, float(np.float32(scale)), _ptr(out))
    return out


def fp8_payload_segments(master_local: np.ndarray, segments):
    """Per segment: amax, scale and codes; returns (codes in compact order, scales list, amax list)."""
    codes, scales, amaxes = [], [], []
    for _, l, n in segments:
        t = master_local[l:l + n]
        a = absmax(t)
        sc = fp8_scale(a)
        amaxes.append(a)
        scales.append(sc)
        codes.append(cast_fp8(t, sc))
    return (np.concatenate(codes) if codes else np.empty(0, np.uint8)), scales, amaxes
