"""Shared plumbing of the GPU parity tests: seeded inputs on host and device, and the
comparison rules.  No arithmetic of the step lives here; expected values come from
``oracle`` only."""
from __future__ import annotations

import dataclasses

import numpy as np

from paper_2311_00257_amd import synth, workloads

REL_TOL = 1e-5          # stated bar: fp32 master/m/v and the gradient norm within 1e-5 relative


def hparams_of(w: workloads.Workload, **over):
    hp = dict(lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, weight_decay=w.weight_decay, step=w.step,
              max_norm=w.max_norm, clip_eps=w.clip_eps)
    hp.update(over)
    return hp


@dataclasses.dataclass
class HostInputs:
    partials: list          # k uint16 arrays (bf16 patterns)
    p: np.ndarray
    m: np.ndarray
    v: np.ndarray


def host_inputs(w: workloads.Workload, index0: int, n: int, k=None, threads: int = 4) -> HostInputs:
    """The workload's streams for global indices index0 .. index0+n-1."""
    k = w.k if k is None else k
    parts = [synth.fill_bf16(w.key(synth.TENSOR_PARTIAL0 + j), index0, n, w.sigma_grad, threads=threads)
             for j in range(k)]
    return HostInputs(parts,
                      synth.fill_f32(w.key(synth.TENSOR_MASTER), index0, n, w.sigma_param, threads=threads),
                      synth.fill_f32(w.key(synth.TENSOR_EXP_AVG), index0, n, w.sigma_m, threads=threads),
                      synth.fill_f32(w.key(synth.TENSOR_EXP_AVG_SQ), index0, n, w.scale_v, absolute=True,
                                     threads=threads))


def to_dev_bf16(bits: np.ndarray, pad_front: int = 0):
    """uint16 patterns -> device int16 tensor; with pad_front > 0 the data starts that many
    elements into a fresh allocation (to shift its alignment)."""
    import torch

    buf = torch.empty(pad_front + bits.size, dtype=torch.int16, device="cuda")
    view = buf[pad_front:]
    view.copy_(torch.from_numpy(bits.view(np.int16)))
    return view


def to_dev_f32(x: np.ndarray, pad_front: int = 0):
    import torch

    buf = torch.empty(pad_front + x.size, dtype=torch.float32, device="cuda")
    view = buf[pad_front:]
    view.copy_(torch.from_numpy(x))
    return view


def dev_bits(t) -> np.ndarray:
    """2-byte device tensor -> uint16 patterns on the host."""
    import torch

    return t.view(torch.int16).cpu().numpy().view(np.uint16)


@dataclasses.dataclass
class GradSum:
    """What a comparison needs to know about a k-term fp32 gradient sum: k and sum_j |g_j[i]| in double,
    the magnitude against which the sum is known."""
    k: int
    abs: np.ndarray


def abs_partials(partials) -> GradSum:
    total = np.zeros(partials[0].size, dtype=np.float64)
    for q in partials:
        total += np.abs(synth.bf16_bits_to_f32(q).astype(np.float64))
    return GradSum(len(partials), total)


ULP = 2.0 ** -24        # unit roundoff of fp32: one correctly rounded operation errs by at most ULP * |result|


def denominators(ref: dict, inp_p, inp_m, hp: dict):
    """Denominators of the relative errors of (master, first moment, second moment): the result itself, or the
    larger operand of its final addition where that addition cancels:
      master        max(|p|, |p' - p|)         (p' = p - step)
      first moment  max(beta1 |m|, (1 - beta1) |g'|)
      second moment v'                         (a sum of non-negative terms: no cancellation)."""
    b1 = float(np.float32(hp["beta1"]))
    gp = np.abs(ref["scale"] * ref["G"])
    den_p = np.maximum(np.abs(inp_p.astype(np.float64)), np.abs(ref["p"] - inp_p))
    den_m = np.maximum(b1 * np.abs(inp_m.astype(np.float64)), (1 - b1) * gp)
    den_v = ref["v"]
    return den_p, den_m, den_v


def rounding_allowances(ref: dict, inp_p, inp_m, hp: dict, abs_g=None):
    """Absolute errors (master, first moment, second moment) that correctly rounded fp32 arithmetic may
    leave, to first order, in places where a relative tolerance on the result cannot cover them:
      e_G  = (k - 1) ULP sum_j |g_j|          a sequential k-term fp32 sum (abs_g: a GradSum; None or k = 1:
                                              the gradient is exact)
      e_g' = |scale| e_G + 2 ULP |g'|         scale rounded to fp32, one product
      e_m  = (1 - beta1) e_g' + 3 ULP tau_m   tau_m = max(beta1 |m|, (1 - beta1) |g'|): the roundings of the
                                              product and of the fused multiply-add are relative to the
                                              operands, not to a result that cancelled
      e_v  = (1 - beta2) (2 |g'| e_g' + e_g'^2) + 3 ULP v'
      e_p  = lr (e_m / bc1) / (sqrt(v_hat) + eps)          the step inherits the first moment's error,
             + lr |u| (e_v / (2 v') + 6 ULP)               the second moment's through the square root,
             + 4 ULP max(|p|, |p' - p|)                    and its own roundings
    These are a few ulps of the operands: far below the relative tolerance wherever nothing cancels."""
    f32 = lambda x: float(np.float32(x))
    b1, b2, lr, eps = f32(hp["beta1"]), f32(hp["beta2"]), f32(hp["lr"]), f32(hp["eps"])
    t = int(hp["step"])
    bc1, bc2 = 1.0 - b1 ** t, 1.0 - b2 ** t
    scale = abs(float(ref["scale"]))
    gp = np.abs(ref["scale"] * ref["G"])
    e_G = 0.0 if abs_g is None else max(abs_g.k - 1, 0) * ULP * abs_g.abs
    e_g = scale * e_G + 2 * ULP * gp
    tau_m = np.maximum(b1 * np.abs(inp_m.astype(np.float64)), (1 - b1) * gp)
    e_m = (1 - b1) * e_g + 3 * ULP * tau_m
    e_v = (1 - b2) * (2 * gp * e_g + e_g * e_g) + 3 * ULP * ref["v"]
    denom = np.sqrt(ref["v"] / bc2) + eps
    denom = np.where(denom > 0, denom, 1.0)
    u = np.abs(ref["m"] / bc1) / denom
    with np.errstate(divide="ignore", invalid="ignore"):
        rel_v = np.where(ref["v"] > 0, e_v / (2.0 * ref["v"]), 0.0)
    den_p = np.maximum(np.abs(inp_p.astype(np.float64)), np.abs(ref["p"] - inp_p))
    e_p = abs(lr) * (e_m / bc1) / denom + abs(lr) * u * (rel_v + 6 * ULP) + 4 * ULP * den_p
    return e_p, e_m, e_v


# share of a workload's elements that may need more than the relative tolerance (see check_state)
RARE = 1e-5


def check_state(got_p, got_m, got_v, ref: dict, inp_p, inp_m, hp: dict, tol: float = REL_TOL, abs_g=None,
                rare=None):
    """fp32 master/m/v against the oracle's doubles: |x - x_ref| <= tol * denominator + rounding allowance
    (see denominators and rounding_allowances).  The allowance matters only where operands cancelled; the
    elements that needed it (error above tol * denominator alone) are counted per quantity in
    stats["extra_p" / "extra_m" / "extra_v"], and with `rare` given their share of the n elements must not
    exceed it (callers pass RARE on the five workloads' own inputs).  The allowance is worked out only for
    those elements.  The strict figures |x - x_ref| / |x_ref| are reported beside them."""
    dens = denominators(ref, inp_p, inp_m, hp)
    stats = {}
    suspects = np.zeros(got_p.size, dtype=bool)
    errs = []
    for name, got, den in zip("pmv", (got_p, got_m, got_v), dens):
        err = np.abs(got.astype(np.float64) - ref[name])
        errs.append(err)
        safe = np.where(den == 0, 1.0, den)
        stats["max_" + name] = float((err / safe).max(initial=0))            # relative to the denominator
        over = err > tol * den
        stats["extra_" + name] = int(np.count_nonzero(over))                   # need the rounding allowance
        suspects |= over
        stats["bad_" + name] = 0
    idx = np.nonzero(suspects)[0]
    if idx.size:
        sub = {key: (val[idx] if isinstance(val, np.ndarray) and val.shape == got_p.shape else val)
               for key, val in ref.items()}
        sub_g = None if abs_g is None else GradSum(abs_g.k, abs_g.abs[idx])
        allow = rounding_allowances(sub, inp_p[idx], inp_m[idx], hp, sub_g)
        for name, err, den, extra in zip("pmv", errs, dens, allow):
            stats["bad_" + name] = int(np.count_nonzero(err[idx] > tol * den[idx] + extra))
    with np.errstate(divide="ignore", invalid="ignore"):
        strict = errs[0] / np.abs(ref["p"])
    stats["strict_max_p"] = float(np.nanmax(strict)) if strict.size else 0.0
    stats["strict_over_tol_p"] = int(np.count_nonzero(strict > tol))
    stats["n"] = int(got_p.size)
    assert stats["bad_p"] == 0 and stats["bad_m"] == 0 and stats["bad_v"] == 0, stats
    if rare is not None:
        most = max(stats["extra_p"], stats["extra_m"], stats["extra_v"])
        assert most <= rare * stats["n"], ("too many elements needed the rounding allowance", stats)
    return stats


def emulate_step_f32(partials, p, m, v, sqnorm, hp):
    """The update as the kernels are documented to compute it, in numpy float32: sequential fp32 sum
    of the partials, scale from the squared norm in double, then per element
        gs = scale*g;  m = fma(b1, m, (1-b1)*gs);  v = fma(b2, v, ((1-b2)*gs)*gs)
        u = (m*rbc1) / (sqrt(v*rbc2) + eps);  p = fma(-lr, fma(wd, p, u), p)
    with every operation correctly rounded once (fma through float64: the product of two float32 is
    exact there).  Not the oracle: a model of the device arithmetic, for a bit-for-bit comparison."""
    f32 = np.float32

    def fma(a, b, c):
        return (np.asarray(a, dtype=np.float64) * np.asarray(b, dtype=np.float64)
                + np.asarray(c, dtype=np.float64)).astype(f32)

    g = synth.bf16_bits_to_f32(partials[0]).astype(f32)
    for q in partials[1:]:
        g = (g + synth.bf16_bits_to_f32(q)).astype(f32)
    b1, b2, lr, eps, wd = (f32(hp[key]) for key in ("beta1", "beta2", "lr", "eps", "weight_decay"))
    scale = 1.0
    if hp["max_norm"] > 0:
        clip = float(f32(hp["max_norm"])) / (np.sqrt(sqnorm) + float(f32(hp["clip_eps"])))
        scale = min(1.0, clip)
    scale = f32(scale)
    omb1, omb2 = f32(1.0 - float(b1)), f32(1.0 - float(b2))
    rbc1 = f32(1.0 / (1.0 - float(b1) ** hp["step"]))
    rbc2 = f32(1.0 / (1.0 - float(b2) ** hp["step"]))
    gs = (scale * g).astype(f32)
    m1 = fma(b1, m, (omb1 * gs).astype(f32))
    v1 = fma(b2, v, ((omb2 * gs).astype(f32) * gs).astype(f32))
    den = (np.sqrt((v1 * rbc2).astype(f32)).astype(f32) + eps).astype(f32)
    u = ((m1 * rbc1).astype(f32) / den).astype(f32)
    p1 = fma(-lr, fma(wd, p, u), p)
    return p1, m1, v1


def check_bf16(got_bits: np.ndarray, ref: dict, inp_p: np.ndarray, tol: float = REL_TOL, inp_m=None,
               hp=None, abs_g=None) -> int:
    """bf16 parameters: identical to bf16(fp32(p')) of the oracle, except where the fp32 tolerance lets p'
    round elsewhere: with delta = what check_state allows the master (tol * max(|p|, |p' - p|), plus the
    rounding allowance when inp_m and hp are given), the shipped value must be the rounding of some value in
    [p' - delta, p' + delta], i.e. lie between bf16(p' - delta) and bf16(p' + delta).  Away from
    cancellation delta is 1/400 of a bf16 step, so this is "exact, or the other neighbour when p' is
    within delta of the midpoint"; where p and the step cancel (p' a million times smaller than its
    operands) it is as wide as the fp32 result is allowed to be.  That the shipped value is exactly bf16
    of the device's own fp32 master is checked separately by the callers.  Returns the number of mismatches."""
    import oracle

    want = ref["p_bf16"]
    bad = np.nonzero(got_bits != want)[0]
    if bad.size == 0:
        return 0
    pp = ref["p"][bad]
    p_in = inp_p[bad].astype(np.float64)
    delta = tol * np.maximum(np.abs(p_in), np.abs(pp - p_in))
    if inp_m is not None and hp is not None:
        delta = delta + rounding_allowances(ref, inp_p, inp_m, hp, abs_g)[0][bad]
    lo = synth.bf16_bits_to_f32(oracle.cast(oracle.round_f32(pp - delta))).astype(np.float64)
    hi = synth.bf16_bits_to_f32(oracle.cast(oracle.round_f32(pp + delta))).astype(np.float64)
    g = synth.bf16_bits_to_f32(got_bits[bad]).astype(np.float64)
    ok = (g >= lo) & (g <= hi)
    assert np.all(ok), "bf16 mismatches outside what the fp32 tolerance allows: %d of %d (first index %d)" % (
        int(np.sum(~ok)), bad.size, int(bad[np.argmin(ok)]))
    return int(bad.size)
