"""GPU test of amsp_grad_sqnorm_static, the entry point that allocates nothing: through the C ABI,
against amsp_grad_sqnorm on the same inputs.  Both run the same kernels in the same order, so the
squared norms must agree bit for bit; the oracle is checked beside them to the stated bar.  Calls come
in pairs, the second on a smaller input, because the library's buffer keeps the previous call's sums."""
import numpy as np
import pytest

import helpers as H
import oracle
from paper_2311_00257_amd import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch

    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2311_00257_amd import binding

    binding.load()
    return binding


def _bits(t) -> int:
    return int(np.float64(t.item()).view(np.uint64))


def _both(B, torch, parts, g32, n, bucket, accumulate, start):
    """(static entry point, existing entry point) results as bit patterns, each from `start`."""
    ws = torch.empty(B.amsp_workspace_bytes() // 8, dtype=torch.float64, device="cuda")
    a = torch.full((1,), start, dtype=torch.float64, device="cuda")
    b = torch.full((1,), start, dtype=torch.float64, device="cuda")
    B.amsp_grad_sqnorm_static(parts, g32, n, a, bucket_elems=bucket, accumulate=accumulate)
    B.amsp_grad_sqnorm(parts, g32, n, b, ws, bucket_elems=bucket, accumulate=accumulate)
    torch.cuda.synchronize()
    return a, b


def test_static_norm_equals_workspace_norm_two_calls_in_a_row(B):
    import torch

    w = workloads.get(1)
    big, small = 9_000_011, 70_003            # the second call is on a smaller input
    inp = H.host_inputs(w, 777, big, k=3)
    dparts = [H.to_dev_bf16(p, pad_front=1) for p in inp.partials]
    mem_before = torch.cuda.memory_allocated()
    for n in (big, small):
        parts = [d[:n] for d in dparts]
        a, b = _both(B, torch, parts, None, n, 0, False, 123.0)
        assert _bits(a) == _bits(b), (n, a.item(), b.item())
        S = oracle.sqnorm(oracle.reduce([p[:n] for p in inp.partials], threads=4))
        assert abs(a.item() - S) <= H.REL_TOL * S
    # the call itself takes no device memory from the allocator the test can see
    d = torch.zeros(1, dtype=torch.float64, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    B.amsp_grad_sqnorm_static([x[:small] for x in dparts], None, small, d)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before and before >= mem_before


@pytest.mark.parametrize("k,bucket", [(1, 0), (8, 0), (2, 300_001), (0, 0), (0, 65_537)])
def test_static_norm_forms(B, k, bucket):
    """Bucketed ranges (many short launches sharing the buffer), the fp32-gradient form, accumulation:
    each as a pair of calls, larger then smaller."""
    import torch

    w = workloads.get(3)
    big, small = 5_000_017, 4_099
    inp = H.host_inputs(w, 31, big, k=max(k, 1))
    if k == 0:
        G = oracle.reduce(inp.partials, threads=4).astype(np.float32)
        g32 = H.to_dev_f32(G, pad_front=3)
        dparts = None
    else:
        g32 = None
        dparts = [H.to_dev_bf16(p) for p in inp.partials]
    for n in (big, small):
        parts = None if dparts is None else [d[:n] for d in dparts]
        g = None if g32 is None else g32[:n]
        for accumulate in (False, True):
            a, b = _both(B, torch, parts, g, n, bucket, accumulate, 0.5)
            assert _bits(a) == _bits(b), (k, bucket, n, accumulate)
        if k == 0:
            S = oracle.sqnorm(G[:n].astype(np.float64))
        else:
            S = oracle.sqnorm(oracle.reduce([p[:n] for p in inp.partials], threads=4))
        assert abs(a.item() - 0.5 - S) <= H.REL_TOL * S


def test_static_norm_empty_and_errors(B):
    import torch

    d = torch.full((1,), 9.0, dtype=torch.float64, device="cuda")
    x = torch.zeros(16, dtype=torch.int16, device="cuda")
    B.amsp_grad_sqnorm_static([x], None, 0, d, accumulate=True)
    torch.cuda.synchronize()
    assert d.item() == 9.0                                   # n == 0 with accumulate: untouched
    B.amsp_grad_sqnorm_static([x], None, 0, d)
    torch.cuda.synchronize()
    assert d.item() == 0.0                                   # n == 0 without: zero
    for args, status in ((([x], None, B.AMSP_STATIC_MAX_ELEMS + 1, d), B.AMSP_ESIZE),
                         (([x] * 33, None, 16, d), B.AMSP_EINVAL),
                         (([x], None, 16, None), B.AMSP_ENULL),
                         ((None, None, 16, d), B.AMSP_ENULL)):
        with pytest.raises(B.AmspError) as ei:
            B.amsp_grad_sqnorm_static(*args)
        assert ei.value.status == status
    torch.cuda.synchronize()
    assert d.item() == 0.0                                   # refused calls enqueue nothing


def test_static_step_in_a_graph(B):
    """What the entry point is for: the whole step (norm pass + fused update) captured in a HIP graph
    with no workspace anywhere, replayed with eager work between the replays, each replay against the
    eager result."""
    import torch

    w = workloads.get(0)
    n = 300_007
    inp = H.host_inputs(w, 5, n)
    hp = H.hparams_of(w)
    dparts = [H.to_dev_bf16(p) for p in inp.partials]
    state0 = [H.to_dev_f32(x) for x in (inp.p, inp.m, inp.v)]

    def run(dst, d_s, out, stream=None):
        B.amsp_grad_sqnorm_static(dparts, None, n, d_s, stream=stream)
        B.amsp_adamw_step_shard(dparts, None, n, dst[0], dst[1], dst[2], out,
                                B.AdamWHparams(d_total_sqnorm=d_s, **hp), stream=stream)

    eager = [x.clone() for x in state0]
    d_e = torch.zeros(1, dtype=torch.float64, device="cuda")
    out_e = torch.zeros(n, dtype=torch.int16, device="cuda")
    run(eager, d_e, out_e)                                   # also the first call on this device: outside capture
    torch.cuda.synchronize()

    work = [x.clone() for x in state0]
    d_g = torch.zeros(1, dtype=torch.float64, device="cuda")
    out_g = torch.zeros(n, dtype=torch.int16, device="cuda")
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            run(work, d_g, out_g, stream=side)
    torch.cuda.synchronize()
    for _ in range(3):
        for dst, src in zip(work, state0):
            dst.copy_(src)                                   # eager work between the replays
        d_g.fill_(-1.0)
        out_g.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert _bits(d_g) == _bits(d_e)
        for a, b in zip(work, eager):
            assert torch.equal(a, b)
        assert torch.equal(out_g, out_e)
