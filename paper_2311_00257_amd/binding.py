"""ctypes binding of the C-ABI library ``libamsp.so`` (declared in ``include/amsp.h``).

Argument marshalling only: every function has the name and meaning of its C counterpart,
takes torch device tensors (or raw integer addresses) where C takes device pointers, and
raises :class:`AmspError` on a non-zero status.  torch supplies device memory and the
stream; all arithmetic runs in the HIP kernels.  There is no fallback: if the library has
not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import dataclasses
import os
from typing import Optional, Sequence

from . import build as _build

AMSP_OK, AMSP_EINVAL, AMSP_ENULL, AMSP_EALIGN, AMSP_EWORKSPACE, AMSP_EDEVICE, AMSP_ENOPLAN, AMSP_ESIZE = \
    0, -1, -2, -3, -4, -5, -6, -7
AMSP_STATIC_MAX_ELEMS = 1 << 34
AMSP_OP_ALLGATHER, AMSP_OP_REDUCESCATTER, AMSP_OP_ALLREDUCE, AMSP_OP_BROADCAST = 0, 1, 2, 3
AMSP_MAX_K = 32

EXPORTS = ("amsp_status_string", "amsp_workspace_bytes", "amsp_reduce_workspace_bytes",
           "amsp_amax_workspace_bytes", "amsp_shard_range", "amsp_reduce_grad_shard", "amsp_grad_sqnorm",
           "amsp_adamw_step_shard", "amsp_cast_param_shard", "amsp_reduce_grad_sqnorm_shard", "amsp_grad_sqnorm_static",
           "amsp_partition_tensors", "amsp_owned_segments", "amsp_reduce_grad_segments", "amsp_grad_sqnorm_segments",
           "amsp_adamw_step_segments", "amsp_cast_param_fp8_shard", "amsp_fp8_payload_segments",
           "amsp_plan_sharding")


class AmspError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: status %d (%s)" % (where, status, amsp_status_string(status)))


class _Segment(ctypes.Structure):
    _fields_ = [("flat_offset", ctypes.c_uint64), ("local_offset", ctypes.c_uint64), ("length", ctypes.c_uint64)]


class _BwSample(ctypes.Structure):
    _fields_ = [("op", ctypes.c_uint32), ("p0", ctypes.c_uint32), ("p1", ctypes.c_uint32),
                ("bytes", ctypes.c_double), ("bytes_per_s", ctypes.c_double)]


class _PlanProblem(ctypes.Structure):
    _fields_ = [("phi", ctypes.c_double), ("layers", ctypes.c_uint32), ("modules_per_layer", ctypes.c_uint32),
                ("module_params", ctypes.POINTER(ctypes.c_double)), ("micro_batches", ctypes.c_uint32),
                ("bucket_bytes", ctypes.c_double), ("gpus_per_node", ctypes.c_uint32), ("nodes", ctypes.c_uint32),
                ("gpu_memory_bytes", ctypes.c_double), ("activation_bytes", ctypes.c_double),
                ("tmp_bytes", ctypes.c_double)]


class _Plan(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint32) for n in ("sp0", "sp1", "sg0", "sg1", "sos0", "sos1")] + \
               [(n, ctypes.c_double) for n in ("t_p", "t_g", "t_os0", "t_os1", "t_comm", "d_modelstate")]


class _Hparams(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float),
                ("eps", ctypes.c_float), ("weight_decay", ctypes.c_float), ("step", ctypes.c_uint32),
                ("max_norm", ctypes.c_float), ("clip_eps", ctypes.c_float),
                ("d_total_sqnorm", ctypes.c_void_p), ("grad_scale", ctypes.c_float)]


@dataclasses.dataclass
class AdamWHparams:
    """Mirror of ``amsp_adamw_hparams``; ``d_total_sqnorm`` is a device double tensor or None."""
    lr: float
    beta1: float
    beta2: float
    eps: float
    weight_decay: float
    step: int
    max_norm: float = 0.0
    clip_eps: float = 1e-6
    d_total_sqnorm: object = None
    grad_scale: float = 1.0


_lib = None


def load() -> ctypes.CDLL:
    """Load ``libamsp.so`` from the package directory; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB_AMSP):
            raise RuntimeError("libamsp.so is not built: run `python -m paper_2311_00257_amd.build` "
                               "(there is no CPU fallback)")
        # torch supplies the device memory these kernels touch, so the library must bind to the
        # HIP runtime torch has loaded: importing torch first makes the dynamic linker reuse it
        # (two HIP runtimes in one process do not see each other's device state).
        import torch  # noqa: F401

        lib = ctypes.CDLL(_build.LIB_AMSP)
        u64, u32, vp, ci = ctypes.c_uint64, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_int
        lib.amsp_status_string.argtypes = [ci]
        lib.amsp_status_string.restype = ctypes.c_char_p
        lib.amsp_workspace_bytes.argtypes = []
        lib.amsp_workspace_bytes.restype = ctypes.c_size_t
        lib.amsp_shard_range.argtypes = [u64, u32, u32, ctypes.POINTER(u64), ctypes.POINTER(u64)]
        lib.amsp_reduce_workspace_bytes.argtypes = [u64, u64]
        lib.amsp_reduce_workspace_bytes.restype = ctypes.c_size_t
        lib.amsp_reduce_grad_shard.argtypes = [vp, u32, u64, u64, vp, ci, vp]
        lib.amsp_reduce_grad_sqnorm_shard.argtypes = [vp, u32, u64, u64, vp, ci, vp, ci, vp, ctypes.c_size_t, vp]
        lib.amsp_grad_sqnorm.argtypes = [vp, u32, vp, u64, u64, vp, ci, vp, ctypes.c_size_t, vp]
        lib.amsp_grad_sqnorm_static.argtypes = [vp, u32, vp, u64, u64, vp, ci, vp]
        lib.amsp_adamw_step_shard.argtypes = [vp, u32, vp, u64, u64, vp, vp, vp, vp, ctypes.POINTER(_Hparams), vp]
        lib.amsp_cast_param_shard.argtypes = [vp, vp, u64, vp]
        pu64, pu32 = ctypes.POINTER(u64), ctypes.POINTER(u32)
        lib.amsp_partition_tensors.argtypes = [pu64, u32, u32, pu32]
        lib.amsp_owned_segments.argtypes = [pu64, pu32, u32, u32, ctypes.POINTER(_Segment), u32, pu32, pu64]
        lib.amsp_grad_sqnorm_segments.argtypes = [vp, u32, u64, ctypes.POINTER(_Segment), u32, vp, ci, vp,
                                                  ctypes.c_size_t, vp]
        lib.amsp_adamw_step_segments.argtypes = [vp, u32, vp, u64, ctypes.POINTER(_Segment), u32, u64, vp, vp, vp,
                                                 vp, vp, vp, ctypes.c_size_t, ctypes.POINTER(_Hparams), vp]
        lib.amsp_reduce_grad_segments.argtypes = [vp, u32, u64, ctypes.POINTER(_Segment), u32, u64, vp, ci, vp]
        lib.amsp_amax_workspace_bytes.argtypes = [u32]
        lib.amsp_amax_workspace_bytes.restype = ctypes.c_size_t
        lib.amsp_cast_param_fp8_shard.argtypes = [vp, u64, vp, vp, vp]
        lib.amsp_fp8_payload_segments.argtypes = [vp, u64, ctypes.POINTER(_Segment), u32, u64, vp, vp, ctypes.c_int,
                                                  vp, vp]
        lib.amsp_plan_sharding.argtypes = [ctypes.POINTER(_PlanProblem), ctypes.POINTER(_BwSample), u32,
                                           ctypes.POINTER(_Plan), pu32]
        for name in EXPORTS[4:]:
            getattr(lib, name).restype = ci
        _lib = lib
    return _lib


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch

        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _partials(partials: Optional[Sequence]):
    if partials is None:
        return None, 0
    k = len(partials)
    arr = (ctypes.c_void_p * max(k, 1))(*[_ptr(p) for p in partials])
    return arr, k


def _check(status: int, where: str) -> None:
    if status != AMSP_OK:
        raise AmspError(status, where)


def amsp_status_string(status: int) -> str:
    return load().amsp_status_string(status).decode()


def amsp_workspace_bytes() -> int:
    return int(load().amsp_workspace_bytes())


def amsp_shard_range(total_elems: int, shard_factor: int, rank: int):
    b, e = ctypes.c_uint64(), ctypes.c_uint64()
    _check(load().amsp_shard_range(total_elems, shard_factor, rank, ctypes.byref(b), ctypes.byref(e)),
           "amsp_shard_range")
    return b.value, e.value


def amsp_reduce_workspace_bytes(n: int, bucket_elems: int = 0) -> int:
    return int(load().amsp_reduce_workspace_bytes(n, bucket_elems))


def _nbytes(t, given: Optional[int]) -> int:
    if given is not None:
        return given
    return 0 if t is None or isinstance(t, int) else t.numel() * t.element_size()


def amsp_reduce_grad_shard(partials, n: int, grad_out, bucket_elems: int = 0, accumulate: bool = False,
                           stream=None) -> None:
    arr, k = _partials(partials)
    _check(load().amsp_reduce_grad_shard(arr, k, n, bucket_elems, _ptr(grad_out), int(accumulate),
                                         _stream(stream)), "amsp_reduce_grad_shard")


def amsp_reduce_grad_sqnorm_shard(partials, n: int, grad_out, d_sqnorm, workspace, bucket_elems: int = 0,
                                  accumulate: bool = False, sqnorm_accumulate: bool = False,
                                  workspace_bytes: Optional[int] = None, stream=None) -> None:
    arr, k = _partials(partials)
    _check(load().amsp_reduce_grad_sqnorm_shard(arr, k, n, bucket_elems, _ptr(grad_out), int(accumulate),
                                                _ptr(d_sqnorm), int(sqnorm_accumulate), _ptr(workspace),
                                                _nbytes(workspace, workspace_bytes), _stream(stream)),
           "amsp_reduce_grad_sqnorm_shard")


def amsp_grad_sqnorm(partials, grad_f32, n: int, d_sqnorm, workspace, bucket_elems: int = 0,
                     accumulate: bool = False, stream=None, workspace_bytes: Optional[int] = None) -> None:
    arr, k = _partials(partials)
    _check(load().amsp_grad_sqnorm(arr, k, _ptr(grad_f32), n, bucket_elems, _ptr(d_sqnorm), int(accumulate),
                                   _ptr(workspace), _nbytes(workspace, workspace_bytes), _stream(stream)),
           "amsp_grad_sqnorm")


def amsp_grad_sqnorm_static(partials, grad_f32, n: int, d_sqnorm, bucket_elems: int = 0, accumulate: bool = False,
                            stream=None) -> None:
    arr, k = _partials(partials)
    _check(load().amsp_grad_sqnorm_static(arr, k, _ptr(grad_f32), n, bucket_elems, _ptr(d_sqnorm), int(accumulate),
                                          _stream(stream)), "amsp_grad_sqnorm_static")


def amsp_adamw_step_shard(partials, grad_f32, n: int, master, exp_avg, exp_avg_sq, param_bf16_out,
                          hp: AdamWHparams, bucket_elems: int = 0, stream=None) -> None:
    arr, k = _partials(partials)
    c = None
    if hp is not None:
        c = _Hparams(hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, hp.step, hp.max_norm, hp.clip_eps,
                     _ptr(hp.d_total_sqnorm), hp.grad_scale)
    _check(load().amsp_adamw_step_shard(arr, k, _ptr(grad_f32), n, bucket_elems, _ptr(master), _ptr(exp_avg),
                                        _ptr(exp_avg_sq), _ptr(param_bf16_out),
                                        ctypes.byref(c) if c is not None else None, _stream(stream)),
           "amsp_adamw_step_shard")


def amsp_cast_param_shard(master, param_bf16_out, n: int, stream=None) -> None:
    _check(load().amsp_cast_param_shard(_ptr(master), _ptr(param_bf16_out), n, _stream(stream)),
           "amsp_cast_param_shard")


# ------------------------------------------------------------------ inter-tensor shards
def _hp_struct(hp: AdamWHparams):
    return _Hparams(hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, hp.step, hp.max_norm, hp.clip_eps,
                    _ptr(hp.d_total_sqnorm), hp.grad_scale)


class SegmentArray:
    """A segment list already laid out as the C array the entry points take: build it once with
    ``marshal_segments`` and pass it wherever a list of (flat_offset, local_offset, length) goes, so
    that a long list is not converted again on every call."""

    def __init__(self, segments):
        self.n = len(segments)
        self.arr = (_Segment * max(self.n, 1))(*[_Segment(*map(int, s)) for s in segments])

    def __len__(self):
        return self.n


def marshal_segments(segments) -> SegmentArray:
    return segments if isinstance(segments, SegmentArray) else SegmentArray(segments)


def _segments(segments):
    a = marshal_segments(segments)
    return a.arr, a.n


def amsp_partition_tensors(tensor_elems: Sequence[int], shard_factor: int):
    """owner index per tensor (list of int)."""
    n = len(tensor_elems)
    sizes = (ctypes.c_uint64 * max(n, 1))(*tensor_elems)
    owner = (ctypes.c_uint32 * max(n, 1))()
    _check(load().amsp_partition_tensors(sizes, n, shard_factor, owner), "amsp_partition_tensors")
    return list(owner[:n])


def amsp_owned_segments(tensor_elems: Sequence[int], owner: Sequence[int], rank: int):
    """([(flat_offset, local_offset, length), ...], local_elems) of `rank`."""
    n = len(tensor_elems)
    sizes = (ctypes.c_uint64 * max(n, 1))(*tensor_elems)
    own = (ctypes.c_uint32 * max(n, 1))(*owner)
    count, local = ctypes.c_uint32(), ctypes.c_uint64()
    _check(load().amsp_owned_segments(sizes, own, n, rank, None, 0, ctypes.byref(count), ctypes.byref(local)),
           "amsp_owned_segments")
    segs = (_Segment * max(count.value, 1))()
    _check(load().amsp_owned_segments(sizes, own, n, rank, segs, count.value, ctypes.byref(count),
                                      ctypes.byref(local)), "amsp_owned_segments")
    return [(s.flat_offset, s.local_offset, s.length) for s in segs[:count.value]], local.value


def amsp_grad_sqnorm_segments(partials_flat, flat_elems: int, segments, d_sqnorm, workspace,
                              accumulate: bool = False, stream=None, workspace_bytes: Optional[int] = None) -> None:
    arr, k = _partials(partials_flat)
    segs, ns = _segments(segments)
    _check(load().amsp_grad_sqnorm_segments(arr, k, flat_elems, segs, ns, _ptr(d_sqnorm), int(accumulate),
                                            _ptr(workspace), _nbytes(workspace, workspace_bytes), _stream(stream)),
           "amsp_grad_sqnorm_segments")


def amsp_adamw_step_segments(partials_flat, flat_elems: int, segments, local_elems: int, master_local,
                             exp_avg_local, exp_avg_sq_local, param_bf16_flat, hp: AdamWHparams, stream=None,
                             d_amax=None, amax_workspace=None, amax_workspace_bytes: Optional[int] = None,
                             grad_f32_local=None) -> None:
    """partials_flat: list of k flat bf16 buffers, or None with grad_f32_local (the k = 0 form)."""
    if partials_flat is None:
        arr, k = None, 0
    else:
        arr, k = _partials(partials_flat)
    segs, ns = _segments(segments)
    c = _hp_struct(hp) if hp is not None else None
    _check(load().amsp_adamw_step_segments(arr, k, _ptr(grad_f32_local), flat_elems, segs, ns, local_elems,
                                           _ptr(master_local), _ptr(exp_avg_local), _ptr(exp_avg_sq_local),
                                           _ptr(param_bf16_flat), _ptr(d_amax), _ptr(amax_workspace),
                                           _nbytes(amax_workspace, amax_workspace_bytes),
                                           ctypes.byref(c) if c is not None else None, _stream(stream)),
           "amsp_adamw_step_segments")


def amsp_reduce_grad_segments(partials_flat, flat_elems: int, segments, local_elems: int, grad_f32_local,
                              accumulate: bool = False, stream=None) -> None:
    arr, k = _partials(partials_flat)
    segs, ns = _segments(segments)
    _check(load().amsp_reduce_grad_segments(arr, k, flat_elems, segs, ns, local_elems, _ptr(grad_f32_local),
                                            int(accumulate), _stream(stream)), "amsp_reduce_grad_segments")


def amsp_amax_workspace_bytes(num_segments: int) -> int:
    return int(load().amsp_amax_workspace_bytes(num_segments))


# ------------------------------------------------------------------ FP8 payload
def amsp_cast_param_fp8_shard(master, n: int, d_scale, param_fp8_out, stream=None) -> None:
    _check(load().amsp_cast_param_fp8_shard(_ptr(master), n, _ptr(d_scale), _ptr(param_fp8_out), _stream(stream)),
           "amsp_cast_param_fp8_shard")


def amsp_fp8_payload_segments(master_local, local_elems: int, segments, flat_elems: int, param_fp8_flat, d_amax,
                              d_scale, stream=None, amax_ready: bool = False) -> None:
    segs, ns = _segments(segments)
    _check(load().amsp_fp8_payload_segments(_ptr(master_local), local_elems, segs, ns, flat_elems,
                                            _ptr(param_fp8_flat), _ptr(d_amax), 1 if amax_ready else 0,
                                            _ptr(d_scale), _stream(stream)),
           "amsp_fp8_payload_segments")


# ------------------------------------------------------------------ sharding planner
def amsp_plan_sharding(phi: float, layers: int, module_params: Sequence[float], micro_batches: int,
                       bucket_bytes: float, gpus_per_node: int, nodes: int, gpu_memory_bytes: float,
                       activation_bytes: float, tmp_bytes: float, table):
    """table: iterable of (op, p0, p1, bytes, bytes_per_s).  Returns (plan dict, feasible_count);
    raises AmspError(AMSP_ENOPLAN) when nothing fits."""
    mods = (ctypes.c_double * max(len(module_params), 1))(*module_params)
    rows = [_BwSample(int(o), int(a), int(b), float(v), float(w)) for (o, a, b, v, w) in table]
    arr = (_BwSample * max(len(rows), 1))(*rows)
    pb = _PlanProblem(phi, layers, len(module_params), mods, micro_batches, bucket_bytes, gpus_per_node, nodes,
                      gpu_memory_bytes, activation_bytes, tmp_bytes)
    best, count = _Plan(), ctypes.c_uint32()
    _check(load().amsp_plan_sharding(ctypes.byref(pb), arr, len(rows), ctypes.byref(best), ctypes.byref(count)),
           "amsp_plan_sharding")
    return (dict(s=(best.sp0, best.sp1, best.sg0, best.sg1, best.sos0, best.sos1), t_p=best.t_p, t_g=best.t_g,
                 t_os0=best.t_os0, t_os1=best.t_os1, t_comm=best.t_comm, d_modelstate=best.d_modelstate),
            count.value)
