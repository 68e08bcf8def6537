#!/usr/bin/env python3
"""Benchmark of the per-GPU model-state step on one MI355X.

A step is one pass of the whole path over one rank's shard, inputs resident in HBM:
    amsp_grad_sqnorm (k bf16 partials -> squared norm)           2k   bytes/element
    amsp_adamw_step_shard (reduce + clip + AdamW + bf16 cast)    2k+26 bytes/element
The other composition of the same steps (reduce with the norm fused in -> fp32 gradient ->
AdamW + cast, 2k+34 bytes/element in all) is timed afterwards and reported as "alt_step".
Default workload: LLaMA-7B at shard factor 8, rank 3, k = 8 (842,301,952 elements).
Prints ONE JSON line: throughput in elements/s, the HBM roofline of the fused kernel from
HIP-event timing of that kernel alone, and the CPU oracle timed on a bounded slice.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=1, help="workload id 0..5 (default 1: LLaMA-7B, factor 8, k = 8)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-alt", action="store_true", help="skip the materialised-gradient composition")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the plain device copy timed for context beside the kernels")
    ap.add_argument("--cpu-sample-elems", type=int, default=512 * 1024 * 1024)
    ap.add_argument("--traffic-file", default=os.path.join(ROOT, "profiles", "adamw_kernel_llama7b_s8r3_k8_hbm_traffic.txt"),
                    help="rocprofv3 --pmc summary holding the fused kernel's measured HBM bytes per launch")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (a kernel of known traffic, for scaling "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    return ap.parse_args()


def ceilings(torch, out, master, n):
    """What plain streaming reaches on this machine in this run, for context beside roofline.frac: the
    runtime's own device-to-device copy of the fp32 master shard (4n bytes read + 4n written), and the
    library's read-only norm pass already timed above.  Boxes differ by a few per cent."""
    scratch = torch.empty_like(master)
    scratch.copy_(master)
    times = []
    for _ in range(7):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        scratch.copy_(master)
        e1.record()
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1))
    del scratch
    copy_ms = sorted(times)[len(times) // 2]
    return {"device_copy": {"GB/s": 8 * n / (copy_ms * 1e-3) / 1e9, "ms": copy_ms, "bytes": 8 * n,
                            "what": "torch copy_ of the fp32 master shard, read + written bytes"},
            "read_only": {"GB/s": out["norm_pass"]["GB/s"], "what": "the norm pass over the k partials"}}


def cpu_baseline(w, begin, sample):
    """The oracle as it stands, timed on the host cores over a slice of the same workload."""
    import oracle
    from paper_2311_00257_amd import synth

    cores = min(len(os.sched_getaffinity(0)), 16)
    parts = [synth.fill_bf16(w.key(synth.TENSOR_PARTIAL0 + j), begin, sample, w.sigma_grad, threads=cores)
             for j in range(w.k)]
    p = synth.fill_f32(w.key(synth.TENSOR_MASTER), begin, sample, w.sigma_param, threads=cores)
    m = synth.fill_f32(w.key(synth.TENSOR_EXP_AVG), begin, sample, w.sigma_m, threads=cores)
    v = synth.fill_f32(w.key(synth.TENSOR_EXP_AVG_SQ), begin, sample, w.scale_v, absolute=True, threads=cores)
    hp = dict(lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, weight_decay=w.weight_decay, step=w.step,
              max_norm=w.max_norm, clip_eps=w.clip_eps)
    res = {}
    for label, th in (("all", cores), ("one", 1)):
        n_run = sample if th > 1 else max(1, sample // 8)
        t0 = time.perf_counter()
        oracle.step([q[:n_run] for q in parts], p[:n_run], m[:n_run], v[:n_run], threads=th, **hp)
        res[label] = n_run / (time.perf_counter() - t0)
    return {"value": res["all"], "unit": "elements/s", "cores": cores, "kind": "oracle",
            "sample": "first %d elements of the %s shard, whole step (reduce, norm, clip, AdamW, cast) in fp64; "
                      "one contiguous chunk per thread" % (sample, w.name),
            "single_thread_value": res["one"]}


def alt_step(args, torch, B, w, n, parts, master, exp_avg, exp_avg_sq, param_bf16, d_sqnorm):
    """The other composition of the same steps, timed after the primary one: amsp_reduce_grad_sqnorm_shard
    writes the fp32 gradient (2k + 4 bytes/element), then amsp_adamw_step_shard on that
    gradient with the bf16 cast (30 bytes/element): 2k + 34 in all instead of 4k + 26."""
    g32 = torch.empty(n, dtype=torch.float32, device="cuda")
    ws = torch.empty(B.amsp_reduce_workspace_bytes(n, w.bucket_elems) // 8, dtype=torch.float64, device="cuda")

    def step(t, ev=None):
        hp = B.AdamWHparams(lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, weight_decay=w.weight_decay,
                            step=t, max_norm=w.max_norm, clip_eps=w.clip_eps, d_total_sqnorm=d_sqnorm)
        if ev:
            ev[0].record()
        B.amsp_reduce_grad_sqnorm_shard(parts, n, g32, d_sqnorm, ws, bucket_elems=w.bucket_elems)
        if ev:
            ev[1].record()
        B.amsp_adamw_step_shard(None, g32, n, master, exp_avg, exp_avg_sq, param_bf16, hp,
                                bucket_elems=w.bucket_elems)
        if ev:
            ev[2].record()

    for i in range(args.warmup):
        step(w.step + i)
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(w.step + args.warmup + i, events[i])
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    red_ms = sum(e[0].elapsed_time(e[1]) for e in events) / args.steps
    upd_ms = sum(e[1].elapsed_time(e[2]) for e in events) / args.steps
    return {"composition": "reduce+norm -> fp32 gradient -> AdamW+cast", "bytes_per_element": 2 * w.k + 34,
            "ms_per_step": ms, "value": n / (ms * 1e-3), "unit": "elements/s",
            "reduce_norm": {"ms": red_ms, "GB/s": (2 * w.k + 4) * n / (red_ms * 1e-3) / 1e9,
                            "bytes_per_element": 2 * w.k + 4},
            "adamw_f32_grad": {"ms": upd_ms, "GB/s": 30 * n / (upd_ms * 1e-3) / 1e9, "bytes_per_element": 30}}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding across GPUs); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2311_00257_amd import binding as B
    from paper_2311_00257_amd import synth, synth_device, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    B.load()
    torch.cuda.set_device(0)
    w = workloads.get(args.config)
    k = w.k
    workspace = torch.empty(B.amsp_workspace_bytes() // 8, dtype=torch.float64, device="cuda")
    d_sqnorm = torch.zeros(1, dtype=torch.float64, device="cuda")

    def hparams(t):
        return B.AdamWHparams(lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, weight_decay=w.weight_decay,
                              step=t, max_norm=w.max_norm, clip_eps=w.clip_eps, d_total_sqnorm=d_sqnorm)

    # ---- inputs resident in HBM before the timed region
    if not w.inter_tensor:
        begin, end = B.amsp_shard_range(w.total_elems, w.shard_factor, w.rank)
        n = end - begin - w.drop_tail
        launches = 1                       # the buckets of one call share a launch (until the grid limit)
        buckets = 1 if not w.bucket_elems else -(-n // w.bucket_elems)
        parts = []
        for j in range(k):
            t = torch.empty(n, dtype=torch.int16, device="cuda")
            synth_device.fill_bf16(t, w.key(synth.TENSOR_PARTIAL0 + j), begin, w.sigma_grad)
            parts.append(t)
        master = torch.empty(n, dtype=torch.float32, device="cuda")
        exp_avg = torch.empty(n, dtype=torch.float32, device="cuda")
        exp_avg_sq = torch.empty(n, dtype=torch.float32, device="cuda")
        synth_device.fill_f32(master, w.key(synth.TENSOR_MASTER), begin, w.sigma_param)
        synth_device.fill_f32(exp_avg, w.key(synth.TENSOR_EXP_AVG), begin, w.sigma_m)
        synth_device.fill_f32(exp_avg_sq, w.key(synth.TENSOR_EXP_AVG_SQ), begin, w.scale_v, absolute=True)
        param_bf16 = torch.empty(n, dtype=torch.int16, device="cuda")

        def norm_pass():
            B.amsp_grad_sqnorm(parts, None, n, d_sqnorm, workspace, bucket_elems=w.bucket_elems)

        def update_pass(t):
            B.amsp_adamw_step_shard(parts, None, n, master, exp_avg, exp_avg_sq, param_bf16, hparams(t),
                                    bucket_elems=w.bucket_elems)
    else:
        # inter-tensor shards: whole tensors chosen greedily, selected from flat whole-model gradient buffers
        sizes, total = w.tensor_sizes, w.total_elems
        owner = B.amsp_partition_tensors(sizes, w.shard_factor)
        segs, n = B.amsp_owned_segments(sizes, owner, w.rank)
        begin, launches, buckets = 0, len(segs), 1
        seg_tuples, segs = segs, B.marshal_segments(segs)      # the C array, built once
        parts = []
        for j in range(k):
            t = torch.empty(total, dtype=torch.int16, device="cuda")
            synth_device.fill_bf16(t, w.key(synth.TENSOR_PARTIAL0 + j), 0, w.sigma_grad)
            parts.append(t)
        master = torch.empty(n, dtype=torch.float32, device="cuda")
        exp_avg = torch.empty(n, dtype=torch.float32, device="cuda")
        exp_avg_sq = torch.empty(n, dtype=torch.float32, device="cuda")
        for f, l, m in seg_tuples:
            synth_device.fill_f32(master[l:l + m], w.key(synth.TENSOR_MASTER), f, w.sigma_param)
            synth_device.fill_f32(exp_avg[l:l + m], w.key(synth.TENSOR_EXP_AVG), f, w.sigma_m)
            synth_device.fill_f32(exp_avg_sq[l:l + m], w.key(synth.TENSOR_EXP_AVG_SQ), f, w.scale_v, absolute=True)
        param_bf16 = torch.empty(total, dtype=torch.int16, device="cuda")

        def norm_pass():
            B.amsp_grad_sqnorm_segments(parts, total, segs, d_sqnorm, workspace)

        def update_pass(t):
            B.amsp_adamw_step_segments(parts, total, segs, n, master, exp_avg, exp_avg_sq, param_bf16, hparams(t))
    torch.cuda.synchronize()

    def step(t, ev=None):
        if ev:
            ev[0].record()
        norm_pass()
        if ev:
            ev[1].record()
        update_pass(t)
        if ev:
            ev[2].record()

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for i in range(args.warmup):
        step(w.step + i)
    torch.cuda.synchronize()

    # ---- timed region: exactly --steps steps, HIP events on the launch stream around each kernel
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(w.step + args.warmup + i, events[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    ms_per_step = wall * 1e3 / args.steps
    norm_ms = sum(e[0].elapsed_time(e[1]) for e in events) / args.steps
    fused_ms = sum(e[1].elapsed_time(e[2]) for e in events) / args.steps
    fused_bytes = w.bytes_per_elem_fused() * n
    achieved = fused_bytes / (fused_ms * 1e-3) / 1e9

    traffic = None
    try:
        fields = dict(line.split(":", 1) for line in open(args.traffic_file) if ":" in line and line[0] != "#")
        if fields.get("workload", "").strip() == w.name:
            traffic = float(fields["hbm_bytes_per_launch"])
    except (OSError, ValueError, KeyError):
        pass

    out = {
        "metric": "model-state elements updated/s per GPU (norm pass + fused reduce/AdamW/bf16-cast step)",
        "value": n / (ms_per_step * 1e-3),
        "unit": "elements/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "elements": n, "k": k, "shard_factor": w.shard_factor, "rank": w.rank,
                   "bucket_elems": w.bucket_elems, "buckets": buckets, "launches_per_pass": launches},
        "roofline": {"bound": "hbm", "kernel": "adamw_kernel<k=%d,bf16 out> (amsp_adamw_step_shard)" % k,
                     "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic,
                     "bytes_per_element": w.bytes_per_elem_fused(), "kernel_ms": fused_ms / launches,
                     "launches": launches},
        "norm_pass": {"ms": norm_ms, "GB/s": w.bytes_per_elem_norm() * n / (norm_ms * 1e-3) / 1e9,
                      "bytes_per_element": w.bytes_per_elem_norm()},
        "whole_step_GBps": (w.bytes_per_elem_fused() + w.bytes_per_elem_norm()) * n / (ms_per_step * 1e-3) / 1e9,
    }
    if w.inter_tensor:
        # the FP8 form of step 4 for inter-tensor shards: per-tensor amax (4 B/elt read), scale, E4M3 codes
        # (4 B/elt read + 1 written), timed on the state the steps above left
        fp8 = torch.empty(w.total_elems, dtype=torch.uint8, device="cuda")
        d_amax = torch.zeros(len(segs), dtype=torch.float32, device="cuda")
        d_scale = torch.zeros(len(segs), dtype=torch.float32, device="cuda")
        for _ in range(2):
            B.amsp_fp8_payload_segments(master, n, segs, w.total_elems, fp8, d_amax, d_scale)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            B.amsp_fp8_payload_segments(master, n, segs, w.total_elems, fp8, d_amax, d_scale)
        e1.record()
        torch.cuda.synchronize()
        fp8_ms = e0.elapsed_time(e1) / args.steps
        out["fp8_payload"] = {"ms": fp8_ms, "GB/s": 9 * n / (fp8_ms * 1e-3) / 1e9, "bytes_per_element": 9,
                              "launches": 2 * len(segs) + 2}
        # the whole step shipping FP8 instead of bf16: norm pass, update with the per-tensor maxima taken
        # inside it and no bf16 output (2k + 24 B/elt), scales and E4M3 codes (4 read + 1 written)
        amax_ws = torch.empty(B.amsp_amax_workspace_bytes(len(segs)) // 4, dtype=torch.int32, device="cuda")

        def fp8_step(t):
            norm_pass()
            B.amsp_adamw_step_segments(parts, total, segs, n, master, exp_avg, exp_avg_sq, None, hparams(t),
                                       d_amax=d_amax, amax_workspace=amax_ws)
            B.amsp_fp8_payload_segments(master, n, segs, w.total_elems, fp8, d_amax, d_scale, amax_ready=True)
        for i in range(2):
            fp8_step(w.step + i)
        e0.record()
        for i in range(args.steps):
            fp8_step(w.step + 2 + i)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        bpe = 2 * k + 2 * k + 24 + 5
        out["fp8_step"] = {"composition": "norm -> AdamW with fused per-tensor amax, no bf16 -> scales + E4M3 codes",
                           "ms_per_step": ms, "value": n / (ms * 1e-3), "unit": "elements/s",
                           "bytes_per_element": bpe, "GB/s": bpe * n / (ms * 1e-3) / 1e9}
        del fp8
    if not args.no_ceilings and not args.calibrate_copy:   # keep the calibration run to one known copy
        out["ceilings"] = ceilings(torch, out, master, n)
    if not args.no_alt and not w.inter_tensor:
        out["alt_step"] = alt_step(args, torch, B, w, n, parts, master, exp_avg, exp_avg_sq, param_bf16, d_sqnorm)
    if not args.no_cpu_baseline:
        del parts, master, exp_avg, exp_avg_sq, param_bf16, norm_pass, update_pass
        out["cpu_baseline"] = cpu_baseline(w, begin, min(args.cpu_sample_elems, n))
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
