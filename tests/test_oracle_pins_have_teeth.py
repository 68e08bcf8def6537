"""Each case plants ONE plausible mistake in a copy of the oracle's C source (a dropped term,
a wrong sign, a wrong index, a wrong rounding rule), builds it on the CPU and runs the pin
tests against the broken build: at least one pin must fail for every mistake.  The real
oracle is restored afterwards."""
import ctypes
import os
import subprocess
import tempfile

import pytest

import oracle
import test_oracle_pins as pins

SRC = open(os.path.join(os.path.dirname(oracle.__file__), "amsp_oracle.c")).read()

MUTATIONS = [
    ("range: every rank charged the full remainder", "uint64_t extra_before = r < rem ? r : rem;", "uint64_t extra_before = rem;"),
    ("range: nobody gets the extra element", "*end = *begin + base + (r < rem ? 1u : 0u);", "*end = *begin + base;"),
    ("reduce: keeps only the last partial", "s += bf16_value(partials[j][i]);", "s = bf16_value(partials[j][i]);"),
    ("reduce: mean instead of sum", "G[i] = s;", "G[i] = s / k;"),
    ("reduce: bf16 widened by the wrong shift", "((uint32_t)b) << 16", "((uint32_t)b) << 15"),
    ("sqnorm: sum of magnitudes", "(long double)G[i] * (long double)G[i]", "fabsl((long double)G[i])"),
    ("clip: norm not rooted", "sqrt(total_sqnorm) + clip_eps", "total_sqnorm + clip_eps"),
    ("clip: scale not capped at one", "return c < 1.0 ? c : 1.0;", "return c;"),
    ("clip: eps dropped", "(sqrt(total_sqnorm) + clip_eps)", "(sqrt(total_sqnorm))"),
    ("adamw: first moment mixes with beta1 twice", "(1.0 - b1) * g;", "b1 * g;"),
    ("adamw: second moment takes g, not g squared", "(1.0 - b2) * g * g;", "(1.0 - b2) * g;"),
    ("adamw: bias correction ignores the step", "1.0 - pow(b1, (double)t)", "1.0 - b1"),
    ("adamw: second bias correction ignores the step", "1.0 - pow(b2, (double)t)", "1.0 - b2"),
    ("adamw: no bias correction of m", "double mhat = m1 / bc1;", "double mhat = m1;"),
    ("adamw: eps inside the root", "sqrt(vhat) + eps", "sqrt(vhat + eps)"),
    ("adamw: weight decay with the wrong sign", "+ wd * pi);", "- wd * pi);"),
    ("adamw: ascent instead of descent", "p_out[i] = pi - lr *", "p_out[i] = pi + lr *"),
    ("adamw: clip scale not applied", "double g = scale * G[i];", "double g = G[i];"),
    ("adamw: decay of the old moment dropped", "b2 * (double)v[i] +", ""),
    ("adamw: moments swapped on output", "m_out[i] = m1;\n        v_out[i] = v1;", "m_out[i] = v1;\n        v_out[i] = m1;"),
    ("cast: ties round up", "u += 0x7FFFu + keep_lsb;", "u += 0x8000u;"),
    ("cast: ties round down", "u += 0x7FFFu + keep_lsb;", "u += 0x7FFFu;"),
    ("cast: truncation", "u += 0x7FFFu + keep_lsb;", ""),
    ("cast: NaN not handled", "if ((u & 0x7FFFFFFFu) > 0x7F800000u)", "if (0)"),
    ("cast: NaN loses its sign", "(((u >> 16) & 0x8000u) | 0x7FC0u)", "(0x7FC0u)"),
    ("e4m3: wrong exponent bias", "return sign | (uint8_t)(((e + 7) << 3) | ((int)r - 8));", "return sign | (uint8_t)(((e + 8) << 3) | ((int)r - 8));"),
    ("e4m3: subnormal spacing of the wrong binade", "if (e < -6) e = -6;", "if (e < -7) e = -7;"),
    ("e4m3: mantissa carry not propagated", "if (r >= 16.0) { r = 8.0; e += 1; }", "if (r >= 16.0) { r = 15.0; }"),
    ("e4m3: no saturation at the tie above 448", "if (a >= 464.0) return sign | 0x7E;", "if (a >= 480.0) return sign | 0x7E;"),
    ("e4m3: truncation instead of nearest", "double r = nearbyint(a / q);", "double r = floor(a / q);"),
    ("e4m3: decode of subnormals off by one binade", "v = ldexpf((float)m, -9);", "v = ldexpf((float)m, -10);"),
    ("fp8: scale maps amax to 240", "return 448.0f / amax;", "return 240.0f / amax;"),
    ("fp8: signed max instead of max magnitude", "float v = fabsf(p[i]);", "float v = p[i];"),
    ("fp8: scale not applied", "volatile float x = p[i] * scale;", "volatile float x = p[i];"),
]

PIN_TESTS = [getattr(pins, n) for n in dir(pins) if n.startswith("test_") and "synth" not in n]


def _run_all_pins(golden_dir):
    """Names of the pin tests that fail against the oracle currently loaded."""
    failed = []
    for fn in PIN_TESTS:
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        arg_sets = [()]
        if marks:
            names = [a.strip() for a in marks[0].args[0].split(",")]
            arg_sets = [v if isinstance(v, tuple) else (v,) for v in marks[0].args[1]]
            arg_sets = [dict(zip(names, v)) for v in arg_sets]
        for args in arg_sets:
            kwargs = dict(args) if isinstance(args, dict) else {}
            if "golden_dir" in fn.__code__.co_varnames[:fn.__code__.co_argcount]:
                kwargs["golden_dir"] = golden_dir
            try:
                fn(**kwargs)
            except AssertionError:
                failed.append(fn.__name__)
                break
            except Exception:           # a broken oracle may also blow up a library call
                failed.append(fn.__name__)
                break
    return failed


def test_unmutated_oracle_passes_this_harness(golden_dir):
    assert _run_all_pins(golden_dir) == []


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(name, old, new, golden_dir):
    assert SRC.count(old) == 1, "mutation target must occur exactly once: %r" % old
    with tempfile.TemporaryDirectory() as tmp:
        c_path, so_path = os.path.join(tmp, "broken.c"), os.path.join(tmp, "libbroken.so")
        open(c_path, "w").write(SRC.replace(old, new))
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-w", "-o", so_path, c_path, "-lm"])
        good = oracle._load()
        oracle._lib = oracle._bind(ctypes.CDLL(so_path))
        try:
            failed = _run_all_pins(golden_dir)
        finally:
            oracle._lib = good
    assert failed, "no pin noticed: " + name


# --------------------------------------------------------------------------- the planner oracle
import types

import test_planner as planner_pins

PLANNER_SRC = open(os.path.join(os.path.dirname(oracle.__file__), "planner.py")).read()

PLANNER_MUTATIONS = [
    ("T_p: AllGather counted once", "t_p += 2 * ag + rs", "t_p += ag + rs"),
    ("T_p: not multiplied by the layers", "t_p *= M * L", "t_p *= M"),
    ("T_g: every micro-batch instead of all but the last", "t_g = (M - 1) * 2 * phi", "t_g = M * 2 * phi"),
    ("T_os0: bucket count ignores s_p", "t_os0 = 2 * phi / (U * sp) * ar_os", "t_os0 = 2 * phi / U * ar_os"),
    ("T_os1: one broadcast instead of s_os/s_p", "t_os1 = so / sp * bc", "t_os1 = bc"),
    ("T_os1: broadcast of the whole model", "coll_time(table, BC, 2 * phi / so,", "coll_time(table, BC, 2 * phi,"),
    ("memory: optimizer states counted as 8 bytes", "+ 12 * phi / so", "+ 8 * phi / so"),
    ("memory: activations ignored", 'c["d_modelstate"] + activation + tmp > gpu_memory', 'c["d_modelstate"] > gpu_memory'),
    ("constraint: s_g free between s_p and s_os", "if (sg0, sg1) != (sp0, sp1) and (sg0, sg1) != (so0, so1):", "if False:"),
    ("constraint: nodes before the node is full", "if any(b > 1 and a != R for a, b in", "if any(False for a, b in"),
    ("constraint: factors need not divide", "if any(R % a for a in (sp0, sg0, so0)) or any(N % a for a in (sp1, sg1, so1)):", "if False:"),
    ("constraint: chain s_p <= s_g <= s_os not enforced", "if not (1 <= sp0 <= sg0 <= so0 <= R and 1 <= sp1 <= sg1 <= so1 <= N):", "if not (1 <= sp0 <= R and 1 <= so0 <= R and 1 <= sp1 <= N and 1 <= so1 <= N):"),
    ("AllReduce mesh: the sharded group instead of its complement", "coll_time(table, AR, U, R // sp0, N // sp1)", "coll_time(table, AR, U, sp0, sp1)"),
    ("interpolation: nearest lower sample", "return w0 if b1 == b0 else w0 + (w1 - w0) * (v - b0) / (b1 - b0)", "return w0"),
    ("one-GPU mesh priced from the table", "if p0 * p1 == 1:\n        return 0.0", "if False:\n        return 0.0"),
    ("tie: last tuple wins", 'if best is None or c["t_comm"] < best["t_comm"]:', 'if best is None or c["t_comm"] <= best["t_comm"]:'),
]

PLANNER_PINS = [getattr(planner_pins, n) for n in dir(planner_pins)
                if n.startswith("test_") and "library" not in n]


def _run_planner_pins(golden_dir):
    failed = []
    for fn in PLANNER_PINS:
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        arg_sets = [{}]
        if marks:
            names = [a.strip() for a in marks[0].args[0].split(",")]
            arg_sets = [dict(zip(names, v if isinstance(v, tuple) else (v,))) for v in marks[0].args[1]]
        for kwargs in arg_sets:
            kwargs = dict(kwargs)
            if "golden_dir" in fn.__code__.co_varnames[:fn.__code__.co_argcount]:
                kwargs["golden_dir"] = golden_dir
            try:
                fn(**kwargs)
            except Exception:
                failed.append(fn.__name__)
                break
    return failed


def test_unmutated_planner_passes_this_harness(golden_dir):
    assert _run_planner_pins(golden_dir) == []


@pytest.mark.parametrize("name,old,new", PLANNER_MUTATIONS, ids=[m[0] for m in PLANNER_MUTATIONS])
def test_planted_planner_mistake_is_caught(name, old, new, golden_dir):
    assert PLANNER_SRC.count(old) == 1, "mutation target must occur exactly once: %r" % old
    broken = types.ModuleType("broken_planner")
    exec(compile(PLANNER_SRC.replace(old, new), "broken_planner.py", "exec"), broken.__dict__)
    good = planner_pins.P
    planner_pins.P = broken
    try:
        failed = _run_planner_pins(golden_dir)
    finally:
        planner_pins.P = good
    assert failed, "no pin noticed: " + name
