"""Calls longer than one launch: a range of more than 2^33 elements is cut on the host into consecutive
launches of at most 2^25 workgroups.  One cast and one fused step of 2^33 + 2^20 + 3 elements (two
launches, the second with a ragged tail), checked against the oracle on windows at the start, on both
sides of the cut, at the end and at seeded places; the cast also against torch's own bf16 conversion
over every element.  Needs 70 GB / 140 GB of device memory."""
import numpy as np
import pytest

import helpers as H
import oracle
from paper_2311_00257_amd import synth, workloads

pytestmark = pytest.mark.gpu

N = (1 << 33) + (1 << 20) + 3
CUT = 1 << 33
WINDOW = 1 << 14


def _windows(seed):
    rng = np.random.default_rng(seed)
    starts = [0, CUT - WINDOW, CUT - WINDOW // 2, CUT, N - WINDOW] + [int(x) for x in rng.integers(0, N - WINDOW, 8)]
    return sorted(starts)


def _need(bytes_needed):
    import torch

    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    if free < bytes_needed + (2 << 30):
        pytest.skip("needs %.0f GB of device memory, %.0f free" % (bytes_needed / 1e9, free / 1e9))


def test_cast_longer_than_one_launch():
    import torch

    from paper_2311_00257_amd import binding as B
    from paper_2311_00257_amd import synth_device

    _need(N * 8 + 128)
    w = workloads.get(2)
    master = torch.empty(N, dtype=torch.float32, device="cuda")
    synth_device.fill_f32(master, w.key(synth.TENSOR_MASTER), 0, w.sigma_param)
    guard = 64
    buf = torch.full((N + 2 * guard,), 0x5A5A, dtype=torch.int16, device="cuda")
    out = buf[guard:guard + N]
    B.amsp_cast_param_shard(master, out, N)
    torch.cuda.synchronize()
    assert bool(torch.all(buf[:guard] == 0x5A5A)) and bool(torch.all(buf[guard + N:] == 0x5A5A))
    for a in _windows(1):
        got = H.dev_bits(out[a:a + WINDOW])
        want = oracle.cast(synth.fill_f32(w.key(synth.TENSOR_MASTER), a, WINDOW, w.sigma_param))
        assert np.array_equal(got, want), a
    # every element: the inputs are finite, where torch's conversion is the same round-to-nearest-even
    step = 1 << 31
    for a in range(0, N, step):
        b = min(N, a + step)
        assert torch.equal(master[a:b].to(torch.bfloat16).view(torch.int16), out[a:b]), a
    print("cast of %d elements in two launches: windows and every element agree" % N, flush=True)


def test_fused_step_longer_than_one_launch():
    import torch

    from paper_2311_00257_amd import binding as B
    from paper_2311_00257_amd import synth_device

    _need(N * 16)
    w = workloads.get(2)                                     # k = 1: one all-reduced gradient buffer
    part = torch.empty(N, dtype=torch.int16, device="cuda")
    synth_device.fill_bf16(part, w.key(synth.TENSOR_PARTIAL0), 0, w.sigma_grad)
    dp = torch.empty(N, dtype=torch.float32, device="cuda")
    dm = torch.empty(N, dtype=torch.float32, device="cuda")
    dv = torch.empty(N, dtype=torch.float32, device="cuda")
    synth_device.fill_f32(dp, w.key(synth.TENSOR_MASTER), 0, w.sigma_param)
    synth_device.fill_f32(dm, w.key(synth.TENSOR_EXP_AVG), 0, w.sigma_m)
    synth_device.fill_f32(dv, w.key(synth.TENSOR_EXP_AVG_SQ), 0, w.scale_v, absolute=True)
    out = torch.empty(N, dtype=torch.int16, device="cuda")
    hp = H.hparams_of(w, max_norm=0.0)                       # a fixed scale: the norm pass is not what is tested here
    B.amsp_adamw_step_shard([part], None, N, dp, dm, dv, out, B.AdamWHparams(grad_scale=0.0078125, **hp))
    torch.cuda.synchronize()
    tally = dict(max_p=0.0, max_m=0.0, max_v=0.0)
    for a in _windows(2):
        inp = H.host_inputs(w, a, WINDOW, threads=8)
        G = oracle.reduce(inp.partials, threads=8)
        p1, m1, v1 = oracle.adamw(G, 0.0078125, inp.p, inp.m, inp.v, lr=hp["lr"], beta1=hp["beta1"], beta2=hp["beta2"],
                                  eps=hp["eps"], weight_decay=hp["weight_decay"], step=hp["step"], threads=8)
        ref = dict(G=G, scale=0.0078125, p=p1, m=m1, v=v1, p_bf16=oracle.cast(oracle.round_f32(p1)))
        sl = slice(a, a + WINDOW)
        gp = dp[sl].cpu().numpy()
        st = H.check_state(gp, dm[sl].cpu().numpy(), dv[sl].cpu().numpy(), ref, inp.p, inp.m, hp,
                           abs_g=H.abs_partials(inp.partials))
        bits = H.dev_bits(out[sl])
        H.check_bf16(bits, ref, inp.p, inp_m=inp.m, hp=hp, abs_g=H.abs_partials(inp.partials))
        assert np.array_equal(bits, oracle.cast(gp))
        for key in tally:
            tally[key] = max(tally[key], st[key])
    print("fused step of %d elements in two launches: %s" % (N, tally), flush=True)
