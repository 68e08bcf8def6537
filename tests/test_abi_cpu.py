"""CPU-only checks of the C-ABI library: it loads, exports every function the header
declares, and its host-side logic (shard ranges, argument validation) behaves as
documented.  Nothing here launches device work."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_2311_00257_amd import binding as B
from paper_2311_00257_amd import build, workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def _built():
    if not build.built():
        build.build_all(verbose=False)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "amsp.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(amsp_[a-z0-9_]+)\s*\(", header))
    assert {"amsp_shard_range", "amsp_reduce_grad_shard", "amsp_grad_sqnorm", "amsp_adamw_step_shard",
            "amsp_cast_param_shard"} <= declared
    lib = B.load()
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert declared == set(B.EXPORTS)
    synth_lib = ctypes.CDLL(build.LIB_SYNTH)
    assert hasattr(synth_lib, "amsp_synth_fill_f32") and hasattr(synth_lib, "amsp_synth_fill_bf16")
    probe_lib = ctypes.CDLL(build.LIB_PROBE)          # bench.py's traffic-only kernels, a library of their own
    assert hasattr(probe_lib, "amsp_probe_traffic") and not hasattr(lib, "amsp_probe_traffic")


def test_stream_placement_helper():
    """layout.staggered_empty: stream j starts (first_index + j) * stagger bytes into an allocation of its
    own, with the length and type asked for; stagger 0 gives plain tensors."""
    import torch

    from paper_2311_00257_amd import layout

    specs = [(1000, torch.float32), (1000, torch.int16), (0, torch.float32), (7, torch.uint8)]
    plain = layout.staggered_empty(specs, stagger=0, device="cpu")
    assert [t.storage_offset() for t in plain] == [0, 0, 0, 0]
    for first in (0, 3):
        views = layout.staggered_empty(specs, first_index=first, device="cpu")
        assert layout.STAGGER_BYTES == 4096
        for j, (t, (n, dtype)) in enumerate(zip(views, specs)):
            assert t.dtype == dtype and t.numel() == n and t.is_contiguous()
            assert t.storage_offset() * t.element_size() == (first + j) * 4096
            assert t.untyped_storage().nbytes() == n * t.element_size() + (first + j) * 4096
        storages = {t.untyped_storage().data_ptr() for t in views}
        assert len(storages) == len(views)                                  # an allocation each
    with pytest.raises(AssertionError):
        layout.staggered_empty(specs, stagger=512, device="cpu")            # not a wave-piece multiple


def _param_types(header: str, name: str):
    """Parameter types of a declaration in the header, names and spacing stripped."""
    m = re.search(r"\b%s\s*\(([^)]*)\)\s*;" % name, header)
    assert m, name
    types = []
    for decl in m.group(1).split(","):
        decl = " ".join(decl.split())
        decl = re.sub(r"\b[A-Za-z_][A-Za-z0-9_]*$", "", decl).strip()      # drop the parameter's name
        types.append(decl.replace(" *", "*").replace("* ", "*"))
    return types


def test_five_base_entry_points_keep_their_listed_signatures():
    """The five calls the boundary names take exactly these parameter types, in this order; everything
    else the library offers lives in entry points of its own."""
    header = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "amsp.h")).read(), flags=re.S)
    P = "const uint16_t*const*"
    want = {
        "amsp_shard_range": ["uint64_t", "uint32_t", "uint32_t", "uint64_t*", "uint64_t*"],
        "amsp_reduce_grad_shard": [P, "uint32_t", "uint64_t", "uint64_t", "float*", "int", "void*"],
        "amsp_grad_sqnorm": [P, "uint32_t", "const float*", "uint64_t", "uint64_t", "double*", "int", "void*",
                             "size_t", "void*"],
        "amsp_adamw_step_shard": [P, "uint32_t", "const float*", "uint64_t", "uint64_t", "float*", "float*",
                                  "float*", "uint16_t*", "const amsp_adamw_hparams*", "void*"],
        "amsp_cast_param_shard": ["const float*", "uint16_t*", "uint64_t", "void*"],
    }
    for name, types in want.items():
        assert _param_types(header, name) == types, (name, _param_types(header, name))


def test_hparams_struct_layout_matches_header():
    # float x5, uint32, float x2, pointer (8-aligned), float, tail padding
    assert B._Hparams.d_total_sqnorm.offset == 32
    assert B._Hparams.grad_scale.offset == 40
    assert ctypes.sizeof(B._Hparams) == 48


def test_status_strings_and_workspace():
    for code in (0, -1, -2, -3, -4, -5):
        assert B.amsp_status_string(code) and "unknown" not in B.amsp_status_string(code)
    assert "unknown" in B.amsp_status_string(-99)
    assert B.amsp_workspace_bytes() >= 8 and B.amsp_workspace_bytes() % 8 == 0


def test_shard_range_bit_exact_against_oracle():
    rng = np.random.default_rng(0)
    cases = [(w.total_elems, w.shard_factor, w.rank) for w in workloads.WORKLOADS]
    cases += [(10, 3, r) for r in range(3)] + [(2, 4, r) for r in range(4)] + [(0, 5, 2), (2**64 - 1, 1000, 999)]
    cases += [(int(rng.integers(0, 2**50)), int(s), int(rng.integers(0, s))) for s in rng.integers(1, 100000, 2000)]
    for total, s, r in cases:
        assert B.amsp_shard_range(total, s, r) == oracle.shard_range(total, s, r)


def test_shard_range_errors():
    for args in ((10, 0, 0), (10, 4, 4), (10, 4, 5)):
        with pytest.raises(B.AmspError) as ei:
            B.amsp_shard_range(*args)
        assert ei.value.status == B.AMSP_EINVAL
    b = ctypes.c_uint64()
    assert B.load().amsp_shard_range(10, 2, 0, None, ctypes.byref(b)) == B.AMSP_ENULL


HP = dict(lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.0, step=1)


def _status(fn, *a, **kw):
    with pytest.raises(B.AmspError) as ei:
        fn(*a, stream=0, **kw)
    return ei.value.status


def test_argument_validation_without_device():
    """All of these must be rejected on the host before any HIP call (fake addresses)."""
    A = 0x10000   # a 16-byte aligned fake address, never dereferenced
    assert _status(B.amsp_cast_param_shard, 0, A, 8) == B.AMSP_ENULL
    assert _status(B.amsp_cast_param_shard, A, 0, 8) == B.AMSP_ENULL
    assert _status(B.amsp_cast_param_shard, A + 2, A, 8) == B.AMSP_EALIGN
    assert _status(B.amsp_cast_param_shard, A, A + 1, 8) == B.AMSP_EALIGN
    B.amsp_cast_param_shard(0, 0, 0, stream=0)                      # n == 0: fine, nothing to do

    assert _status(B.amsp_reduce_grad_shard, [], 8, A) == B.AMSP_EINVAL
    assert _status(B.amsp_reduce_grad_shard, [A] * 33, 8, A) == B.AMSP_EINVAL
    assert _status(B.amsp_reduce_grad_shard, [A, 0], 8, A) == B.AMSP_ENULL
    assert _status(B.amsp_reduce_grad_shard, [A, A + 1], 8, A) == B.AMSP_EALIGN
    assert _status(B.amsp_reduce_grad_shard, [A], 8, 0) == B.AMSP_ENULL
    assert _status(B.amsp_reduce_grad_shard, [A], 8, A + 2) == B.AMSP_EALIGN
    B.amsp_reduce_grad_shard([A], 0, 0, stream=0)
    need = B.amsp_reduce_workspace_bytes(1 << 20, 0)
    assert need >= 8 * (1 << 20) // 4096
    # the block sums of all buckets lie side by side: 1024 buckets need (about) 1024 times one bucket's share
    many = B.amsp_reduce_workspace_bytes(1 << 30, 1 << 20)
    assert 1024 * (need - 256 * 8) <= many - 256 * 8 <= 1024 * need
    # a ragged last bucket and tiny buckets are covered too (never less than one slot per 256 elements of a launch)
    assert B.amsp_reduce_workspace_bytes(1000, 300) >= 8 * (3 * 2 + 1)
    assert _status(B.amsp_reduce_grad_sqnorm_shard, [A], 1 << 20, A, A, None) == B.AMSP_ENULL
    assert _status(B.amsp_reduce_grad_sqnorm_shard, [A], 1 << 20, A, 0, A, workspace_bytes=need) == B.AMSP_ENULL
    assert _status(B.amsp_reduce_grad_sqnorm_shard, [A], 1 << 20, A, A + 4, A, workspace_bytes=need) == B.AMSP_EALIGN
    assert _status(B.amsp_reduce_grad_sqnorm_shard, [A], 1 << 20, A, A, A, workspace_bytes=need - 8) == B.AMSP_EWORKSPACE
    assert _status(B.amsp_reduce_grad_sqnorm_shard, [], 8, A, A, A, workspace_bytes=need) == B.AMSP_EINVAL

    ws = B.amsp_workspace_bytes()
    assert _status(B.amsp_grad_sqnorm, [A], None, 8, 0, A, workspace_bytes=ws) == B.AMSP_ENULL
    assert _status(B.amsp_grad_sqnorm, [A], None, 8, A, 0, workspace_bytes=ws) == B.AMSP_ENULL
    assert _status(B.amsp_grad_sqnorm, [A], None, 8, A + 4, A, workspace_bytes=ws) == B.AMSP_EALIGN
    assert _status(B.amsp_grad_sqnorm, [A], None, 8, A, A, workspace_bytes=ws - 1) == B.AMSP_EWORKSPACE
    assert _status(B.amsp_grad_sqnorm, None, None, 8, A, A, workspace_bytes=ws) == B.AMSP_ENULL
    assert _status(B.amsp_grad_sqnorm, None, A + 2, 8, A, A, workspace_bytes=ws) == B.AMSP_EALIGN
    assert _status(B.amsp_grad_sqnorm, [A] * 40, None, 8, A, A, workspace_bytes=ws) == B.AMSP_EINVAL

    hp = B.AdamWHparams(**HP)
    assert _status(B.amsp_adamw_step_shard, [A], None, 8, A, A, A, A, None) == B.AMSP_ENULL
    assert _status(B.amsp_adamw_step_shard, [A], None, 8, 0, A, A, A, hp) == B.AMSP_ENULL
    assert _status(B.amsp_adamw_step_shard, None, None, 8, A, A, A, A, hp) == B.AMSP_ENULL
    assert _status(B.amsp_adamw_step_shard, [A], None, 8, A, A + 2, A, A, hp) == B.AMSP_EALIGN
    assert _status(B.amsp_adamw_step_shard, [A], None, 8, A, A, A, A + 1, hp) == B.AMSP_EALIGN
    for bad in (dict(step=0), dict(lr=float("inf")), dict(beta1=1.0), dict(beta2=-0.1), dict(eps=-1e-8),
                dict(weight_decay=float("nan")), dict(max_norm=float("nan")), dict(grad_scale=float("inf"))):
        assert _status(B.amsp_adamw_step_shard, [A], None, 8, A, A, A, A,
                       B.AdamWHparams(**dict(HP, **bad))) == B.AMSP_EINVAL
    B.amsp_adamw_step_shard([A], None, 0, 0, 0, 0, 0, hp, stream=0)      # n == 0


def test_partition_and_segments_bit_exact_against_oracle():
    rng = np.random.default_rng(3)
    cases = [(w.tensor_sizes, s) for w in workloads.WORKLOADS for s in (1, 3, 8, 16)]
    cases += [([int(x) for x in rng.integers(0, 10**9, int(rng.integers(0, 300)))], int(rng.integers(1, 40)))
              for _ in range(50)]
    for sizes, s in cases:
        owner = B.amsp_partition_tensors(sizes, s)
        assert owner == oracle.partition_tensors(sizes, s)
        for r in sorted({0, s - 1, s // 2}):
            segs, local = B.amsp_owned_segments(sizes, owner, r)
            assert segs == oracle.owned_segments(sizes, owner, r)
            assert local == sum(n for _, _, n in segs)
    with pytest.raises(B.AmspError) as ei:
        B.amsp_partition_tensors([1, 2], 0)
    assert ei.value.status == B.AMSP_EINVAL


def test_segment_validation_without_device():
    A = 0x10000
    hp = B.AdamWHparams(**HP)
    ws = B.amsp_workspace_bytes()
    # a segment that runs past the flat buffer or past the local buffers is refused before any launch
    for segs in ([(90, 0, 20)], [(0, 90, 20)], [(2**63, 0, 2**63)], [(0, 0, 10), (95, 10, 10)]):
        with pytest.raises(B.AmspError) as ei:
            B.amsp_adamw_step_segments([A], 100, segs, 100, A, A, A, A, hp, stream=0)
        assert ei.value.status == B.AMSP_EINVAL
    with pytest.raises(B.AmspError) as ei:
        B.amsp_grad_sqnorm_segments([A], 100, [(95, 0, 10)], A, A, stream=0, workspace_bytes=ws)
    assert ei.value.status == B.AMSP_EINVAL
    with pytest.raises(B.AmspError) as ei:
        B.amsp_adamw_step_segments([A], 100, [(0, 0, 10)], 100, 0, A, A, A, hp, stream=0)
    assert ei.value.status == B.AMSP_ENULL
    B.amsp_adamw_step_segments([A], 100, [], 0, 0, 0, 0, 0, hp, stream=0)          # owns nothing: fine
    # the forms through a compact fp32 gradient
    with pytest.raises(B.AmspError) as ei:
        B.amsp_reduce_grad_segments([A], 100, [(95, 0, 10)], 100, A, stream=0)
    assert ei.value.status == B.AMSP_EINVAL
    with pytest.raises(B.AmspError) as ei:
        B.amsp_reduce_grad_segments([A], 100, [(0, 0, 10)], 100, 0, stream=0)
    assert ei.value.status == B.AMSP_ENULL
    with pytest.raises(B.AmspError) as ei:
        B.amsp_reduce_grad_segments([A], 100, [(0, 0, 10)], 100, A + 2, stream=0)
    assert ei.value.status == B.AMSP_EALIGN
    B.amsp_reduce_grad_segments([A], 100, [], 0, 0, stream=0)
    with pytest.raises(B.AmspError) as ei:                   # k = 0 without a gradient buffer
        B.amsp_adamw_step_segments(None, 100, [(0, 0, 10)], 100, A, A, A, A, hp, stream=0)
    assert ei.value.status == B.AMSP_ENULL
    with pytest.raises(B.AmspError) as ei:
        B.amsp_adamw_step_segments(None, 100, [(0, 0, 10)], 100, A, A, A, A, hp, stream=0, grad_f32_local=A + 2)
    assert ei.value.status == B.AMSP_EALIGN
    # per-segment maxima asked for: the workspace is checked before anything is enqueued
    need = B.amsp_amax_workspace_bytes(3)
    assert need == 3 * B.amsp_amax_workspace_bytes(1) > 0 and B.amsp_amax_workspace_bytes(0) == 0
    three = [(0, 0, 10), (20, 10, 10), (40, 20, 10)]
    for kw, status in ((dict(amax_workspace=None), B.AMSP_ENULL),
                       (dict(amax_workspace=A + 2, amax_workspace_bytes=need), B.AMSP_EALIGN),
                       (dict(amax_workspace=A, amax_workspace_bytes=need - 4), B.AMSP_EWORKSPACE)):
        with pytest.raises(B.AmspError) as ei:
            B.amsp_adamw_step_segments([A], 100, three, 100, A, A, A, A, hp, stream=0, d_amax=A, **kw)
        assert ei.value.status == status
    with pytest.raises(B.AmspError) as ei:
        B.amsp_fp8_payload_segments(A, 100, [(95, 0, 10)], 100, A, A, A, stream=0)
    assert ei.value.status == B.AMSP_EINVAL
    with pytest.raises(B.AmspError) as ei:
        B.amsp_fp8_payload_segments(A, 100, [(0, 0, 10)], 100, A, 0, A, stream=0)
    assert ei.value.status == B.AMSP_ENULL
    with pytest.raises(B.AmspError) as ei:
        B.amsp_cast_param_fp8_shard(A, 10, 0, A, stream=0)
    assert ei.value.status == B.AMSP_ENULL
    B.amsp_cast_param_fp8_shard(0, 0, 0, 0, stream=0)


def test_product_package_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2311_00257_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".c", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "amsp_oracle" not in text, f


def test_header_is_plain_c_and_links_against_the_library(tmp_path):
    """include/amsp.h compiles as C99 with gcc (no C++ in the boundary), and a C program that only
    calls the host-side entry points links against libamsp.so and gets the documented answers."""
    import subprocess

    src = tmp_path / "abi_check.c"
    src.write_text(r'''
#include <stdio.h>
#include "amsp.h"
int main(void) {
    uint64_t b = 0, e = 0;
    if (amsp_shard_range(10, 3, 1, &b, &e) != AMSP_OK || b != 4 || e != 7) return 1;
    if (amsp_shard_range(10, 0, 0, &b, &e) != AMSP_EINVAL) return 2;
    if (amsp_workspace_bytes() == 0 || amsp_reduce_workspace_bytes(1u << 20, 0) == 0) return 3;
    uint64_t sizes[4] = {5, 3, 3, 1};
    uint32_t owner[4];
    if (amsp_partition_tensors(sizes, 4, 2, owner) != AMSP_OK) return 4;
    if (owner[0] != 0 || owner[1] != 1 || owner[2] != 1 || owner[3] != 0) return 5;
    amsp_adamw_hparams hp;
    if (sizeof hp != 48) return 6;
    printf("%s\n", amsp_status_string(AMSP_EWORKSPACE));
    return 0;
}
''')
    exe = tmp_path / "abi_check"
    lib_dir = os.path.dirname(build.LIB_AMSP)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe), "-L", lib_dir, "-lamsp", "-Wl,-rpath," + lib_dir], check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=60)
    assert out.returncode == 0, (out.returncode, out.stderr[-500:])
    assert "workspace" in out.stdout


def test_library_sources_keep_their_promises():
    """The header promises that no entry point allocates, frees or synchronises, and the kernels are
    built without packed-fp32 instructions: checked on the sources the library is built from."""
    csrc = os.path.join(ROOT, "paper_2311_00257_amd", "csrc")
    text = ""
    for name in ("amsp_kernels.hip", "amsp_device.h", "amsp_geometry.h", "amsp_planner.cpp"):
        text += open(os.path.join(csrc, name)).read()
    for banned in ("hipMalloc", "hipFree", "hipMemset", "hipMemcpy", "hipDeviceSynchronize", "hipStreamSynchronize",
                   "hipHostRegister", "hipStreamCreate", "hipEventSynchronize"):
        assert banned not in text, banned
    # no process-global knobs in the shipped library: the environment is read only under the sweep macro
    kernels = open(os.path.join(csrc, "amsp_kernels.hip")).read()
    outside = re.sub(r"#ifdef AMSP_TUNING.*?#else", "", kernels, flags=re.S)
    assert "getenv" not in outside and "getenv" not in text.replace(kernels, "")
    assert "AMSP_TUNING" not in open(os.path.join(ROOT, "paper_2311_00257_amd", "build.py")).read()
    flags = open(os.path.join(ROOT, "paper_2311_00257_amd", "build.py")).read()
    assert '"-target-feature", "-Xclang", "-packed-fp32-ops"' in flags and "gfx950" in flags
