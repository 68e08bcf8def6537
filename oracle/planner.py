"""Oracle of the sharding planner (Section V-B): the integer program written out as an
exhaustive search over EVERY tuple (s_p^0, s_p^1, s_g^0, s_g^1, s_os^0, s_os^1) in
[1..R] x [1..N] per component, each tuple tested against every constraint as the paper
states it, no pruning.  TEST INFRASTRUCTURE ONLY; pure Python.

Cost model (Section IV; FP16/BF16 model states, 2 bytes per parameter and gradient):
  t(o, v, p0 x p1) = v / w(o, v, p0 x p1), w from the profiled table, linear in v between
      the profiled sizes, the end values outside them (Section IV-A); a 1 x 1 mesh costs 0
  T_p    = M L sum_i ( 2 t(AG, 2 Phi_i, s_p) + t(RS, 2 Phi_i, s_p) )                (IV-C.1)
  T_os^0 = 2 Phi / (U s_p) * t(AR, U, s_dp/s_p)                                     (IV-C.2)
  T_os^1 = s_os / s_p * t(BC, 2 Phi / s_os, s_os/s_p)                               (IV-C.2)
  T_g    = (M - 1) 2 Phi / (U s_p) * t(AR, U, s_g/s_p)                              (IV-C.3)
  D_modelstate = 2 Phi/s_p + 2 Phi/s_g + 12 Phi/s_os;  + activations + temporaries  (IV-D)
Constraints: Eq. (2) memory; (3)(4) 1 <= s_p <= s_g <= s_os <= s_dp per mesh dimension;
(5)(6) each factor divides s_dp in its dimension; (7) a component spans nodes only once it
spans the whole node; s_g in {s_p, s_os} (IV-C.3).  s_dp^0 = R, s_dp^1 = N (Table IV note).
Readings where the paper is silent: a mesh absent from the table makes a tuple unusable;
ties keep the first tuple in lexicographic order.
"""
from __future__ import annotations

import itertools

AG, RS, AR, BC = 0, 1, 2, 3


def bandwidth(table, op, v, p0, p1):
    """table: iterable of (op, p0, p1, bytes, bytes_per_s).  None if the mesh was not profiled."""
    pts = sorted((b, w) for (o, a, c, b, w) in table if o == op and a == p0 and c == p1)
    if not pts:
        return None
    if v <= pts[0][0]:
        return pts[0][1]
    if v >= pts[-1][0]:
        return pts[-1][1]
    for (b0, w0), (b1, w1) in zip(pts, pts[1:]):
        if b0 <= v <= b1:
            return w0 if b1 == b0 else w0 + (w1 - w0) * (v - b0) / (b1 - b0)
    raise AssertionError


def coll_time(table, op, v, p0, p1):
    if p0 * p1 == 1:
        return 0.0
    w = bandwidth(table, op, v, p0, p1)
    return None if w is None else v / w


def constraints_hold(s, R, N):
    """Eq. (3)-(7) and s_g in {s_p, s_os}, as stated."""
    sp0, sp1, sg0, sg1, so0, so1 = s
    if not (1 <= sp0 <= sg0 <= so0 <= R and 1 <= sp1 <= sg1 <= so1 <= N):             # (3) (4)
        return False
    if any(R % a for a in (sp0, sg0, so0)) or any(N % a for a in (sp1, sg1, so1)):   # (5) (6)
        return False
    if any(b > 1 and a != R for a, b in ((sp0, sp1), (sg0, sg1), (so0, so1))):       # (7)
        return False
    if (sg0, sg1) != (sp0, sp1) and (sg0, sg1) != (so0, so1):                         # s_g in {s_p, s_os}
        return False
    return True


def evaluate(s, phi, layers, module_params, micro_batches, bucket_bytes, R, N, table):
    """Times and model-state memory of one tuple, or None if a collective cannot be priced."""
    sp0, sp1, sg0, sg1, so0, so1 = s
    M, L, U = micro_batches, layers, bucket_bytes
    sp, sg, so = sp0 * sp1, sg0 * sg1, so0 * so1
    d_ms = 2 * phi / sp + 2 * phi / sg + 12 * phi / so
    parts = []
    t_p = 0.0
    for phi_i in module_params:
        ag = coll_time(table, AG, 2 * phi_i, sp0, sp1)
        rs = coll_time(table, RS, 2 * phi_i, sp0, sp1)
        parts += [ag, rs]
        if ag is not None and rs is not None:
            t_p += 2 * ag + rs
    t_p *= M * L
    ar_os = coll_time(table, AR, U, R // sp0, N // sp1)
    bc = coll_time(table, BC, 2 * phi / so, so0 // sp0, so1 // sp1)
    ar_g = coll_time(table, AR, U, sg0 // sp0, sg1 // sp1)
    if any(x is None for x in parts + [ar_os, bc, ar_g]):
        return None
    t_os0 = 2 * phi / (U * sp) * ar_os
    t_os1 = so / sp * bc
    t_g = (M - 1) * 2 * phi / (U * sp) * ar_g
    return dict(s=tuple(s), t_p=t_p, t_g=t_g, t_os0=t_os0, t_os1=t_os1, t_comm=t_p + t_g + t_os0 + t_os1,
                d_modelstate=d_ms)


def plan(phi, layers, module_params, micro_batches, bucket_bytes, R, N, gpu_memory, activation, tmp, table):
    """Returns (best, feasible_count); best is a dict or None."""
    best, count = None, 0
    rng0, rng1 = range(1, R + 1), range(1, N + 1)
    for s in itertools.product(rng0, rng1, rng0, rng1, rng0, rng1):
        if not constraints_hold(s, R, N):
            continue
        c = evaluate(s, phi, layers, module_params, micro_batches, bucket_bytes, R, N, table)
        if c is None or c["d_modelstate"] + activation + tmp > gpu_memory:           # (2)
            continue
        count += 1
        if best is None or c["t_comm"] < best["t_comm"]:
            best = c
    return best, count
