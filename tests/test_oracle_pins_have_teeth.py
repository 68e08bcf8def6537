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
