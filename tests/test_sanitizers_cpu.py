"""Host-side sanitizer tier (CPU only): the plain-C oracle, the sharding planner and the range-geometry
checker built with gcc's -fsanitize=address,undefined, aborting on the first report, and run on the same
cases the ordinary tests use.  Nothing here touches the GPU or the HIP kernels (there is no device-side
sanitizer on the test machines); what it covers is the host code the parity claims lean on."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]
ORACLE_C = os.path.join(ROOT, "oracle", "amsp_oracle.c")
CSRC = os.path.join(ROOT, "paper_2311_00257_amd", "csrc")


def _clean(res):
    assert res.returncode == 0, (res.returncode, res.stdout[-1500:], res.stderr[-3000:])
    for word in ("runtime error", "AddressSanitizer", "LeakSanitizer", "UndefinedBehaviorSanitizer"):
        assert word not in res.stderr, res.stderr[-3000:]


def test_oracle_under_address_and_undefined_sanitizers(tmp_path):
    """Every function of the C oracle on seeded inputs at sizes 0 ... 4097 with exactly-sized heap buffers,
    k up to 32, wild bit patterns included: the instrumented build reports nothing and prints the same
    checksums as the plain one."""
    driver = os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c")
    plain, inst = str(tmp_path / "plain"), str(tmp_path / "inst")
    subprocess.run(["gcc", "-O2", "-std=c11", "-Wall", "-o", plain, driver, ORACLE_C, "-lm"], check=True)
    subprocess.run(["gcc", *SAN, "-std=c11", "-Wall", "-o", inst, driver, ORACLE_C, "-lm"], check=True)
    a = subprocess.run([plain], capture_output=True, text=True, timeout=120)
    b = subprocess.run([inst], capture_output=True, text=True, timeout=300)
    _clean(a)
    _clean(b)
    assert a.stdout == b.stdout and a.stdout.count("\n") == 8 * 5 + 1


def test_oracle_pins_under_the_undefined_behaviour_sanitizer():
    """The whole pin suite of the oracle once more, in a fresh interpreter, against a build of the oracle
    instrumented with -fsanitize=undefined (that runtime loads into an uninstrumented Python; the address
    sanitizer's does not, hence the stand-alone driver above)."""
    env = dict(os.environ, AMSP_ORACLE_UBSAN="1")
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                          os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                         capture_output=True, text=True, timeout=900, env=env, cwd=ROOT)
    assert res.returncode == 0, (res.stdout[-3000:], res.stderr[-3000:])
    assert "runtime error" not in res.stderr and "runtime error" not in res.stdout
    assert " passed" in res.stdout and "failed" not in res.stdout
    assert os.path.exists(os.path.join(ROOT, "oracle", "libamsp_oracle_ubsan.so"))


def test_geometry_checker_under_sanitizers(tmp_path):
    """The checker that emulates every block and lane of the kernels' range geometry, instrumented: the
    shared header does no out-of-bounds or undefined arithmetic on the host side either."""
    exe = str(tmp_path / "geometry_check")
    subprocess.run(["g++", *SAN, "-std=c++17", "-Wall", "-I", CSRC, "-o", exe,
                    os.path.join(ROOT, "tests", "geometry_check.cpp")], check=True)
    res = subprocess.run([exe], capture_output=True, text=True, timeout=900)
    _clean(res)
    assert res.stdout.startswith("ok 60000")


def test_planner_under_sanitizers_equals_the_oracle(tmp_path):
    """csrc/amsp_planner.cpp compiled with the sanitizers into a stand-alone program, on the 60 seeded
    problems of the planner tests: same plans as the exhaustive Python oracle, to the last bit of the
    tuple and 1e-12 of the times, and nothing reported."""
    from oracle import planner as P

    from test_planner import random_problems

    exe = str(tmp_path / "planner_driver")
    subprocess.run(["g++", *SAN, "-std=c++17", "-Wall", "-I", os.path.join(ROOT, "include"), "-o", exe,
                    os.path.join(ROOT, "tests", "sanitize", "planner_driver.cpp"),
                    os.path.join(CSRC, "amsp_planner.cpp")], check=True)
    problems = list(random_problems())
    text = []
    for phi, layers, mods, M, U, R, N, mem, act, tmp, table in problems:
        text.append("%r %d %d %r %d %d %r %r %r %d %d" % (phi, layers, M, U, R, N, mem, act, tmp, len(mods), len(table)))
        text.append(" ".join(repr(x) for x in mods))
        text += ["%d %d %d %r %r" % (op, p0, p1, float(v), float(bw)) for op, p0, p1, v, bw in table]
    res = subprocess.run([exe], input="\n".join(text) + "\n", capture_output=True, text=True, timeout=900)
    _clean(res)
    lines = res.stdout.strip().split("\n")
    assert len(lines) == len(problems)
    planned = 0
    for args, line in zip(problems, lines):
        want, count = P.plan(*args)
        f = line.split()
        if want is None:
            assert f == ["status", "-6"], line              # AMSP_ENOPLAN
            continue
        assert f[1] == "0" and tuple(int(x) for x in f[2:8]) == want["s"] and int(f[14]) == count
        got = [float.fromhex(x) for x in f[8:14]]
        for value, key in zip(got, ("t_p", "t_g", "t_os0", "t_os1", "t_comm", "d_modelstate")):
            assert value == pytest.approx(want[key], rel=1e-12, abs=0.0)
        planned += 1
    assert planned >= 30
