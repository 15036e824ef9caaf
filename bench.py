#!/usr/bin/env python3
"""Benchmark of the activation-compression hot path on one MI355X.

A step is one pass of the whole path (statistics -> DS-ACIQ directed search -> clip +
quantize + pack -> unpack + dequantize) over the ViT-Base stage-boundary tensor
64x197x768 fp32, once per bitwidth in {2,3,4,6,8,16} (six passes), with every result kept
on the device (no host round trip inside the step).  Inputs are synthetic (seeded mixture of
Laplace and Gaussian values with scaled outliers), resident in HBM before the timed region;
passes rotate over 16 distinct input/output buffer sets (> 600 MB) so that the tensor is not
served from the 256 MB Infinity Cache left warm by the previous pass.

Prints ONE JSON line.  `value` is activation bytes entering the path per second.
`roofline` describes the kernel that dominates the step (the directed-search kernel, bound by
plain vector ALU work); `roofline_pack` / `roofline_unpack` / `roofline_stats` describe the
HBM-bound kernels.  `cpu_baseline` is the CPU oracle timed on a bounded sample of the same
workload on this machine's host cores.
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

HBM_PEAK_GBS = 8000.0                  # MI355X HBM3E, published
# Vector-ALU peak for the search kernel's operation mix.  Published vector peaks: fp32 157.3 TFLOP/s
# and fp64 78.6 TFLOP/s, i.e. (an FMA counting two flops) 78.64e12 fp32 and 39.32e12 fp64 lane
# operations per second (256 CUs x 2.4 GHz x 128 resp. 64 lanes).  Per element and candidate the
# search does 6 fp32 operations (clamp, subtract, multiply, round, fma, subtract) and 2 fp64-class
# ones (convert, fma): at peak that takes 6/78.64e12 + 2/39.32e12 s, so 8 operations run at
# 8 / (6/78.64 + 2/39.32) = 62.9e12 lane operations per second at best.
SEARCH_LANEOPS_PER_ELEM_CAND = 8       # algorithmic vector operations per element and candidate
VALU_PEAK_TLANEOPS = 8.0 / (6.0 / 78.64 + 2.0 / 39.32)
NBUF = 16

# HBM traffic per launch (bytes) from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on this workload, scaled by
# what the same counters read for plain device copies of the tensor in the same run (summary and
# commands: profiles/hbm_traffic_C2_fp32.txt).  pack / unpack: mean over the six bitwidths.
TRAFFIC_BYTES = {"search": 89.74e6, "pack": 46.61e6, "unpack": 46.75e6, "stats": 77.96e6}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-large", action="store_true", help="skip the 151M-element bf16 tensor leg")
    ap.add_argument("--no-c4", action="store_true", help="skip the microbatch-stream leg (32x257x1280 fp32 per microbatch)")
    ap.add_argument("--only-small", action="store_true",
                    help="run only the 1x197x768 leg and print its figures (for a profile of the small-tensor path)")
    ap.add_argument("--no-small", action="store_true",
                    help="skip the 1x197x768 leg (it launches the same kernels on a small tensor, which would mix "
                         "into a profiler's per-kernel averages)")
    ap.add_argument("--kernel-reps", type=int, default=64, help="back-to-back launches per kernel timing")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (tensors shard by microbatch with no exchange); "
              "use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2211_04515_amd as qp
    import synth_inputs as si

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    qp.lib()
    torch.cuda.set_device(0)
    if args.only_small:
        def reps_small(fn, R=args.kernel_reps):
            for r in range(4):
                fn(r)
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for r in range(R):
                fn(r)
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) * 1e3 / R
        print(json.dumps({"small_tensor_fp32": small_tensor_leg(qp, si, torch, reps_small)}))
        return 0
    name = "C2"
    bits_set = si.CONFIG_BITS[name]
    x_host = si.make_config(name)
    n = x_host.size
    in_bytes = n * 4

    xs = [torch.from_numpy(x_host).cuda() for _ in range(NBUF)]
    ys = [torch.empty(n, dtype=torch.float32, device="cuda") for _ in range(NBUF)]
    packs = {b: [qp.alloc_packed(n, b) for _ in range(NBUF)] for b in bits_set}
    ws = qp.alloc_workspace(n)
    qdev = ws.data_ptr() + qp.qp_ws_offset(qp.QP_WS_QPARAMS)
    ev = lambda: torch.cuda.Event(enable_timing=True)

    counter = [0]

    def one_pass(bits, timers=None):
        i = counter[0] % NBUF
        counter[0] += 1
        if timers is None:
            qp.qp_compress_async(xs[i], bits, ws, packs[bits][i])
            qp.qp_unpack_dequant_dev(packs[bits][i], bits, qdev, ys[i])
            return
        e = [ev() for _ in range(5)]
        e[0].record()
        qp.qp_stats_async(xs[i], ws)
        e[1].record()
        qp.qp_dsaciq_search_async(xs[i], bits, ws)
        e[2].record()
        qp.qp_quant_pack_dev(xs[i], bits, qdev, packs[bits][i])
        e[3].record()
        qp.qp_unpack_dequant_dev(packs[bits][i], bits, qdev, ys[i])
        e[4].record()
        timers.append((bits, e))

    def step(timers=None):
        for b in bits_set:
            one_pass(b, timers)

    # four plain device copies of the tensor: under a rocprofv3 counter run these calibrate what
    # FETCH_SIZE / WRITE_SIZE read for a kernel that moves a known number of bytes
    for i in range(4):
        ys[i].copy_(xs[i])
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # timed region: exactly `steps` steps of the fused device-resident path, nothing else on the stream
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = len(bits_set) * in_bytes / (ms_per_step * 1e-3) / 1e9

    # the same `steps` steps again with a HIP event between the stages of every pass (this costs a few
    # microseconds per pass and one extra small launch, so it is kept out of `value`)
    timers = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(timers)
    torch.cuda.synchronize()
    ms_per_step_instrumented = (time.perf_counter() - t0) * 1e3 / args.steps

    # stage durations from the HIP events of the instrumented repetition (torch's current stream, which is
    # the stream the kernels are launched on)
    stage = {"stats": [], "search": [], "pack": [], "unpack": []}
    for bits, e in timers:
        for k, s in enumerate(("stats", "search", "pack", "unpack")):
            stage[s].append(e[k].elapsed_time(e[k + 1]) * 1e3)
    mean = lambda v: float(sum(v) / len(v))
    search_us = mean(stage["search"])       # setup kernel (a few microseconds) + search kernel
    search_ops = SEARCH_LANEOPS_PER_ELEM_CAND * 101 * n
    roofline = {"kernel": "k_search_mse<fp32> (+ k_search_setup)", "bound": "alu",
                "achieved": search_ops / (search_us * 1e-6) / 1e12, "peak": VALU_PEAK_TLANEOPS,
                "unit": "Tlaneop/s", "frac": None, "traffic": TRAFFIC_BYTES["search"],
                "us_per_launch": search_us,
                "timed": "HIP events around every search launch in an instrumented repetition of the timed steps"}
    roofline["frac"] = roofline["achieved"] / roofline["peak"]

    # the HBM-bound kernels: short (about 10 us), so an event pair per launch would add a fifth to
    # them; time kernel_reps back-to-back launches over rotating buffers between two events
    def timed_reps(fn):
        R = args.kernel_reps
        for r in range(4):
            fn(r)
        torch.cuda.synchronize()
        a, b = ev(), ev()
        a.record()
        for r in range(R):
            fn(r)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e3 / R

    per_bits = {}
    for b in bits_set:
        q = qp.read_ws(ws, qp.QP_WS_QPARAMS, qp.qp_qparams_t)
        q = qp.qp_make_qparams((q.lo + q.hi) / 2, (q.hi - q.lo) / 2, b, n)
        tp = timed_reps(lambda r: qp.qp_quant_pack(xs[r % NBUF], q, packs[b][r % NBUF]))
        tu = timed_reps(lambda r: qp.qp_unpack_dequant(packs[b][r % NBUF], q, ys[r % NBUF]))
        byts = in_bytes + n * b / 8
        per_bits[str(b)] = {"pack_us": tp, "pack_GBs": byts / tp / 1e3, "unpack_us": tu, "unpack_GBs": byts / tu / 1e3}
    ts = timed_reps(lambda r: qp.qp_stats_async(xs[r % NBUF], ws))
    # second reference line beside the nominal 8 TB/s: what a plain device-to-device copy of a tensor of this
    # size reaches under the same timing (one launch per tensor, rotating buffers)
    tcopy = timed_reps(lambda r: ys[r % NBUF].copy_(xs[(r + 1) % NBUF]))
    copy_ref = {"kernel": "torch device-to-device copy (not part of the path)", "bytes": 2 * in_bytes, "us": tcopy,
                "GBs": 2 * in_bytes / tcopy / 1e3}
    # the histogram-fit reading of Eq. 1 works on the 2048-bin histogram only (no tensor pass)
    th = timed_reps(lambda r: qp.qp_dsaciq_hist_search_async(4, ws))
    # beyond the paper: coarse-to-fine sweep (stride 10: 11 + 19 candidates instead of 101), same winner on one-valley curves
    c2f = qp.qp_default_search_cfg()
    c2f.flags, c2f.coarse_stride = qp.QP_SEARCH_COARSE_TO_FINE, 10
    qp.qp_stats_async(xs[0], ws)
    tc = timed_reps(lambda r: qp.qp_dsaciq_search_async(xs[r % NBUF], 4, ws, cfg=c2f))
    # the deployment policy the paper reports (directed search active at 2 and 4 bit only): the same six-bitwidth
    # step with the search skipped above 4 bit; reported beside the headline, which searches at every bitwidth
    pol = qp.qp_default_search_cfg()
    pol.flags = qp.QP_SEARCH_LOW_BITS_ONLY

    def policy_step(r):
        for b in bits_set:
            qp.qp_compress_async(xs[r % NBUF], b, ws, packs[b][r % NBUF], cfg=pol)
            qp.qp_unpack_dequant_dev(packs[b][r % NBUF], b, qdev, ys[r % NBUF])
    tpol = timed_reps(policy_step)

    def hbm(kernel, byts, us, key):
        a = byts / us / 1e3
        return {"kernel": kernel, "bound": "hbm", "achieved": a, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": a / HBM_PEAK_GBS, "traffic": TRAFFIC_BYTES[key], "us_per_launch": us,
                "timed": f"{args.kernel_reps} back-to-back launches over {NBUF} rotating buffer sets between two HIP events"}

    # headline for pack / unpack: the mean over the six bitwidths of the workload
    pack_bytes = sum(in_bytes + n * b / 8 for b in bits_set)
    pack_us = sum(per_bits[str(b)]["pack_us"] for b in bits_set)
    unpack_us = sum(per_bits[str(b)]["unpack_us"] for b in bits_set)
    r_pack = hbm("k_quant_pack<k,fp32>, k in {2,3,4,6,8,16}", pack_bytes / len(bits_set), pack_us / len(bits_set), "pack")
    r_unpack = hbm("k_unpack_dequant<k>, k in {2,3,4,6,8,16}", pack_bytes / len(bits_set), unpack_us / len(bits_set), "unpack")
    r_stats = hbm("k_stats_pass1 + k_stats_pass2", 2 * in_bytes, ts, "stats")

    # the large bf16 tensor (256x577x1024, 302 MB in: larger than the Infinity Cache by itself):
    # the HBM-honest reading of the same two kernels, kernel-only
    large = None
    if not args.no_large:
        del xs, ys, packs
        torch.cuda.empty_cache()
        large = large_tensor_leg(qp, si, torch, timed_reps, args.kernel_reps)

    # one image's activations (1x197x768 fp32): the whole sender path per tensor, launch-bound
    small = None if args.no_small else small_tensor_leg(qp, si, torch, timed_reps)

    # a stream of microbatches whose bitwidth follows a bandwidth trace: sustained time per microbatch
    c4 = None
    if not args.no_c4 and not args.no_large:
        c4 = c4_stream_leg(qp, si, torch)

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(x_host, bits_set)

    out = {
        "metric": "activation GB/s quantize+pack & unpack+dequant (% HBM peak); DS-ACIQ us/tensor",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "C2: ViT-Base stage boundary 64x197x768 fp32, 70% Laplace(0,0.4)/30% N(0.1,1) + 0.05% outliers x30, "
                               "full path (stats, DS-ACIQ t=100, pack, unpack) once per bitwidth in {2,3,4,6,8,16}",
                   "elements": n, "bitwidths": list(bits_set), "passes_per_step": len(bits_set), "buffers_rotated": NBUF},
        "ms_per_step_instrumented": ms_per_step_instrumented,
        "stage_us": {k: mean(v) for k, v in stage.items()},
        "dsaciq_us_per_tensor": search_us,
        "dsaciq_histogram_fit_us_per_tensor": th,
        "dsaciq_coarse_to_fine_us_per_tensor": tc,
        "step_with_search_at_2_to_4_bit_only": {"ms_per_step": tpol / 1e3, "GBs": len(bits_set) * in_bytes / tpol / 1e3},
        "roofline": roofline, "roofline_pack": r_pack, "roofline_unpack": r_unpack, "roofline_stats": r_stats,
        "hbm_copy_reference": copy_ref,
        "per_bitwidth": per_bits,
        "large_tensor_bf16": large,
        "small_tensor_fp32": small,
        "microbatch_stream_fp32": c4,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))
    return 0


def large_tensor_leg(qp, si, torch, timed_reps, reps):
    """quantize+pack and unpack+dequantize on the 256x577x1024 bf16 tensor (Student-t, df 3, x0.5)."""
    h = si.make_config("C5")
    n = h.size
    nb = 3
    xs = [torch.from_numpy(h.view("int16").copy()).cuda().view(torch.bfloat16) for _ in range(nb)]
    ys = [torch.empty(n, dtype=torch.float32, device="cuda") for _ in range(nb)]
    ws = qp.alloc_workspace(n)
    st = qp.qp_stats(xs[0], ws)
    out = {"elements": n, "input": "bf16", "buffers_rotated": nb, "stats_us": None}
    out["stats_us"] = timed_reps(lambda r: qp.qp_stats_async(xs[r % nb], ws))
    # a bf16 tensor of this size goes through its value table: one read of the tensor (not two passes)
    out["stats_GBs"] = n * 2 / out["stats_us"] / 1e3
    tcopy = timed_reps(lambda r: ys[(r + 1) % nb].copy_(ys[r % nb]))
    out["hbm_copy_reference_GBs"] = 2 * n * 4 / tcopy / 1e3   # plain device-to-device copy of the fp32 output tensor
    for b in si.CONFIG_BITS["C5"]:
        packs = [qp.alloc_packed(n, b) for _ in range(nb)]
        res, q = qp.qp_dsaciq_search(xs[0], st, b, ws)
        tp = timed_reps(lambda r: qp.qp_quant_pack(xs[r % nb], q, packs[r % nb]))
        tu = timed_reps(lambda r: qp.qp_unpack_dequant(packs[r % nb], q, ys[r % nb]))
        ts = timed_reps(lambda r: qp.qp_dsaciq_search_async(xs[r % nb], b, ws)) if b == 4 else None
        bp, bu = n * 2 + n * b / 8, n * 4 + n * b / 8
        out[str(b)] = {"pack_us": tp, "pack_GBs": bp / tp / 1e3, "pack_frac_hbm": bp / tp / 1e3 / HBM_PEAK_GBS,
                       "unpack_us": tu, "unpack_GBs": bu / tu / 1e3, "unpack_frac_hbm": bu / tu / 1e3 / HBM_PEAK_GBS}
        if ts:
            out["dsaciq_us_per_tensor"] = ts
            # the whole sender path (statistics, search, quantize+pack) per tensor, device-resident parameters
            out["sender_path_us_per_tensor"] = timed_reps(lambda r: qp.qp_compress_async(xs[r % nb], b, ws, packs[r % nb]))
        del packs
    return out


def c4_stream_leg(qp, si, torch, n_mb=48):
    """Sender path + receiver per microbatch (32x257x1280 fp32, 42 MB), back to back on one stream, over a ring of
    eight unit-Laplace buffers scaled per microbatch; the bitwidth of each microbatch follows the seeded bandwidth
    trace.  All inputs are resident before the timed region."""
    n = si.numel("C4")
    stream = si.c4_stream(n_mb)
    ring = [torch.from_numpy(si.unit_laplace(n, 100 + b)).cuda() for b in range(8)]
    xs = [ring[buf] * b_m for (buf, b_m, bw, bits) in stream]          # 48 x 42 MB, all distinct
    packs = {k: qp.alloc_packed(n, k) for k in sorted({s[3] for s in stream})}
    ws = qp.alloc_workspace(n)
    y = torch.empty(n, dtype=torch.float32, device="cuda")
    qdev = ws.data_ptr() + qp.qp_ws_offset(qp.QP_WS_QPARAMS)

    def run():
        for x, (_, _, _, bits) in zip(xs, stream):
            qp.qp_compress_async(x, bits, ws, packs[bits])
            qp.qp_unpack_dequant_dev(packs[bits], bits, qdev, y)

    run()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    run()
    b.record()
    torch.cuda.synchronize()
    us = a.elapsed_time(b) * 1e3 / n_mb
    hist = {}
    for s_ in stream:
        hist[str(s_[3])] = hist.get(str(s_[3]), 0) + 1
    return {"elements_per_microbatch": n, "microbatches": n_mb, "bitwidths_used": hist, "us_per_microbatch": us,
            "activation_GBs": n * 4 / us / 1e3,
            "timed": "statistics, DS-ACIQ (t = 100), quantize+pack, unpack+dequantize per microbatch, one stream, two HIP events"}


def small_tensor_leg(qp, si, torch, timed_reps):
    """Sender path (statistics, DS-ACIQ t = 100, quantize+pack) and its search alone on the 1x197x768 tensor."""
    x = si.make_config("C1")
    n = x.size
    nb = 4
    xs = [torch.from_numpy(x).cuda() for _ in range(nb)]
    ws = qp.alloc_workspace(n)
    packed = qp.alloc_packed(n, 4)
    qp.qp_stats(xs[0], ws)
    t_search = timed_reps(lambda r: qp.qp_dsaciq_search_async(xs[r % nb], 4, ws))
    t_send = timed_reps(lambda r: qp.qp_compress_async(xs[r % nb], 4, ws, packed))
    return {"elements": n, "bits": 4, "dsaciq_us_per_tensor": t_search, "sender_path_us_per_tensor": t_send,
            "timed": "back-to-back calls on one stream between two HIP events"}


def cpu_baseline(x_host, bits_set):
    """The oracle as it stands (single thread, never tuned), on the first quarter of the tensor."""
    from oracle import qp_oracle as orc
    sample = x_host[: x_host.size // 4]
    t0 = time.perf_counter()
    rc, st = orc.stats(sample)
    for b in bits_set:
        res, q, _ = orc.dsaciq_search(sample, st, b, 100)
        codes = orc.quantize(sample, q)
        stream = orc.pack(codes, b)
        y = orc.dequantize(orc.unpack(stream, sample.size, b), q)
    dt = time.perf_counter() - t0
    return {"value": len(bits_set) * sample.size * 4 / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"first quarter of the tensor ({sample.size} elements), all six bitwidths, {dt:.1f} s of CPU time",
            "seconds": dt}


if __name__ == "__main__":
    sys.exit(main())
