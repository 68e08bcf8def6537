"""The range geometry of the kernels (head / vectors / tail, buckets sharing a launch, the alignment
levels) checked exhaustively on the CPU: the header the kernels and the host code share is compiled
as plain C++ into a checker that emulates every block and lane of 60,000 random launches."""
import os
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "tests", "geometry_check.cpp")
HEADER = os.path.join(ROOT, "paper_2311_00257_amd", "csrc", "amsp_geometry.h")


def _run_checker(header_text=None):
    with tempfile.TemporaryDirectory() as tmp:
        inc = os.path.join(tmp, "inc")
        os.mkdir(inc)
        if header_text is None:
            shutil.copy(HEADER, inc)
        else:
            with open(os.path.join(inc, "amsp_geometry.h"), "w") as f:
                f.write(header_text)
        exe = os.path.join(tmp, "geometry_check")
        subprocess.run(["g++", "-O2", "-std=c++17", "-Wall", "-Werror", "-I", inc, "-o", exe, SRC], check=True)
        return subprocess.run([exe], capture_output=True, text=True, timeout=300)


def test_every_element_once_and_every_vector_access_aligned():
    out = _run_checker()
    assert out.returncode == 0, out.stdout[-2000:]
    assert out.stdout.startswith("ok 60000"), out.stdout[-500:]


# The checker has teeth: each of these plausible slips in the header makes it fail.
MUTATIONS = [
    ("head of a bucket ignores where the bucket starts",
     "const uint32_t head = (bk.h0 - (uint32_t)off) & bk.mask;", "const uint32_t head = bk.h0 & bk.mask;"),
    ("head of a bucket added instead of subtracted",
     "const uint32_t head = (bk.h0 - (uint32_t)off) & bk.mask;", "const uint32_t head = (bk.h0 + (uint32_t)off) & bk.mask;"),
    ("last bucket as long as the others",
     "const uint64_t len = left < bk.bucket_elems ? left : bk.bucket_elems;", "const uint64_t len = left < bk.bucket_elems ? bk.bucket_elems : bk.bucket_elems;"),
    ("one block too few per bucket",
     "(uint32_t)(bucket_elems / ((uint64_t)kWaveLanes * vec * rows) + 1)};", "(uint32_t)(bucket_elems / ((uint64_t)kWaveLanes * vec * rows))};"),
    ("blocks per bucket forget the vectors per lane",
     "(uint32_t)(bucket_elems / ((uint64_t)kWaveLanes * vec * rows) + 1)};", "(uint32_t)(bucket_elems / ((uint64_t)kWaveLanes * vec) + 1)};"),
    ("blocks per bucket count the vectors per lane twice",
     "(uint32_t)(bucket_elems / ((uint64_t)kWaveLanes * vec * rows) + 1)};", "(uint32_t)(bucket_elems / ((uint64_t)kWaveLanes * vec * rows * rows) + 1)};"),
    ("tail elements start one vector early",
     "(uint64_t)s.head + s.nvec * (uint64_t)vec + (t - s.head);", "(uint64_t)s.head + (s.nvec - 1) * (uint64_t)vec + (t - s.head);"),
    ("short bucket keeps its aligned head",
     "s.head = (uint32_t)len;\n            s.nvec = 0;", "s.head = head;\n            s.nvec = 0;"),
    ("wave alignment asks for a line only",
     "if (level == kAlignWave) return (uintptr_t)kWaveLanes * vec * elem;", "if (level == kAlignWave) return 128;"),
    ("vector alignment of 2-byte streams forgotten",
     "return (uintptr_t)vec * elem < 16 ? (uintptr_t)vec * elem : 16;", "return elem;"),
    ("period of the line level taken from the widest element",
     "if (st[i].elem < smallest) smallest = st[i].elem;", "if (st[i].elem > smallest) smallest = st[i].elem;"),
    ("norm pass: a trip's pieces not counted into the block's start",
     "uint64_t v = (uint64_t)block * (kWaveLanes * U) + lane;", "uint64_t v = (uint64_t)block * kWaveLanes + lane;"),
    ("norm pass: the grid advances by one piece per trip",
     "v += (uint64_t)U * row) full(v);", "v += row) full(v);"),
    ("norm pass: a full trip taken when only its first piece is inside",
     "for (; v + (uint64_t)(U - 1) * kWaveLanes < nvec;", "for (; v < nvec;"),
    ("long range: the last piece as long as the others",
     "const int rc = f(begin + off, n - off < limit ? n - off : limit);", "const int rc = f(begin + off, limit);"),
    ("long range: pieces overlap by one element",
     "for (uint64_t off = 0; off < n; off += limit) {", "for (uint64_t off = 0; off < n; off += limit - 1) {"),
    ("norm pass: the partial last trip dropped",
     "if (U > 1 && v < nvec) part(v);", "if (U > 1 && v + kWaveLanes < nvec) part(v);"),
    ("norm pass: a partial trip after a trip that was full",
     "if (U > 1 && v < nvec) part(v);", "if (U > 1 && v < nvec + (uint64_t)U * row) part(v - (v >= (uint64_t)U * row ? (uint64_t)U * row : 0));"),
]


@pytest.mark.parametrize("what,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_checker_catches_planted_slips(what, old, new):
    text = open(HEADER).read()
    old, new = old.replace("\\n", "\n"), new.replace("\\n", "\n")
    assert text.count(old) == 1, "mutation target not found exactly once: " + what
    out = _run_checker(text.replace(old, new))
    assert out.returncode != 0 and "FAIL" in out.stdout, what
