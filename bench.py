#!/usr/bin/env python3
"""Benchmark of the activation-compression hot path on one MI355X.

A step is one pass of the whole path (statistics -> DS-ACIQ directed search -> clip +
quantize + pack -> unpack + dequantize) over the ViT-Base stage-boundary tensor
64x197x768 fp32 (C2: the configuration the metric is quoted on), once per bitwidth in
{2,3,4,6,8,16} (six passes), with every result kept on the device (no host round trip inside
the step).  Inputs are synthetic (seeded mixture of Laplace and Gaussian values with scaled
outliers), resident in HBM before the timed region; passes rotate over 16 distinct
input/output buffer sets (> 600 MB) so that the tensor is not served from the 256 MB
Infinity Cache left warm by the previous pass.  The six passes are independent jobs and are
issued round-robin over `--streams` HIP streams (default 3, default priority, a workspace
each), so that the HBM-bound steps of one pass run beside the ALU-bound search of another;
`one_stream` repeats the timed steps with everything on one stream.

Prints ONE JSON line.  `value` is activation bytes entering the path per second.
`roofline` describes the kernel that dominates the step (the directed-search kernel, bound by
plain vector ALU work); `roofline_pack` / `roofline_unpack` / `roofline_stats` describe the
HBM-bound kernels.  The other configurations ride in the same line, each with roofline-shaped
entries of its own: `c3_vit_large_fp32` (64x197x1024 post-GELU, cands_per_round 32),
`large_tensor_bf16` (C5: 256x577x1024 bf16, the largest, HBM-honest by itself),
`microbatch_stream_fp32` (C4: 500 microbatches of 32x257x1280 whose bitwidth follows a
bandwidth trace) and `small_tensor_fp32` (C1: one image, launch-bound; eager and replayed from
a HIP graph).  `cpu_baseline` is the CPU oracle timed on a bounded sample of the C2 workload on
this machine's host cores, single-threaded and with the harness spreading it over the cores.

--legs picks a subset, e.g. `--legs c5` for a profile of the bf16 kernels alone (the timed step is the c2 leg).
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
PREHEAT_S = 0.05                       # of the timed step's own work before the warm-up steps, see c2_leg
ALL_LEGS = ("c2", "c3", "c5", "c1", "c4", "cpu")

# HBM traffic per launch as a multiple of the kernel's algorithmic bytes, from rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE runs of this file, each scaled by what the same counter reads for plain device copies of known
# size inside the same run.  These are calibration constants copied from the tracked summaries named here,
# not measured by this process: a changed kernel shows in them only when those summaries are regenerated.
TRAFFIC_RATIO = {
    # profiles/hbm_traffic_C2_fp32.txt
    "c2_search_bytes": 88.29e6, "c2_pack": 1.0002, "c2_unpack": 1.0033, "c2_stats": 1.0062,
    # profiles/hbm_traffic_C5_bf16.txt
    "c5_value_hist": 1.0094, "c5_pack": 1.0001, "c5_unpack": 1.0022,
}
TRAFFIC_SOURCE = {"c2": "profiles/hbm_traffic_C2_fp32.txt", "c5": "profiles/hbm_traffic_C5_bf16.txt"}


COLD_BYTES = 600e6     # every stream of a per-kernel timing rotates over at least this many bytes of distinct buffers


def cold_count(nbytes, at_least):
    """Buffers of nbytes to rotate over so that this stream alone exceeds the 256 MB Infinity Cache more than twice:
    a packed stream of a few megabytes would otherwise be served from that cache on every repetition (on the 302 MB
    bf16 tensor, three rotating 4-bit payloads of 76 MB fit it and unpack read them at 0.90 of the HBM peak; with the
    payloads cold it does not)."""
    return max(at_least, int(-(-COLD_BYTES // nbytes)))


def cold_payloads(qp, torch, x, q, n, bits, at_least):
    """count distinct packed buffers holding the payload of x under q."""
    first = qp.alloc_packed(n, bits)
    qp.qp_quant_pack(x, q, first)
    out = [first]
    for _ in range(cold_count(first.numel(), at_least) - 1):
        out.append(first.clone())
    return out


def hbm_entry(kernel, alg_bytes, us, traffic_ratio, source, timed):
    a = alg_bytes / us / 1e3
    return {"kernel": kernel, "bound": "hbm", "achieved": a, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": a / HBM_PEAK_GBS, "algorithmic_bytes": alg_bytes,
            "traffic": None if traffic_ratio is None else alg_bytes * traffic_ratio,
            "traffic_source": source, "us_per_launch": us, "timed": timed}


def alu_entry(kernel, n, ncand, us, traffic, timed):
    ops = SEARCH_LANEOPS_PER_ELEM_CAND * ncand * n
    a = ops / (us * 1e-6) / 1e12
    return {"kernel": kernel, "bound": "alu", "achieved": a, "peak": VALU_PEAK_TLANEOPS, "unit": "Tlaneop/s",
            "frac": a / VALU_PEAK_TLANEOPS, "algorithmic_laneops": ops, "traffic": traffic, "us_per_launch": us,
            "timed": timed}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20,
                    help="untimed steps before the timed ones (after a pause on the host the GPU needs some tens of milliseconds "
                         "of work to reach its sustained clock: 3 steps left the first timed steps 6 %% slow)")
    ap.add_argument("--legs", default=",".join(ALL_LEGS),
                    help="comma-separated subset of " + ",".join(ALL_LEGS) + " (default: all).  The timed step is the "
                         "c2 leg; without it only the chosen legs run and `value` is null (for profiles of one leg)")
    ap.add_argument("--kernel-reps", type=int, default=64, help="back-to-back launches per kernel timing")
    ap.add_argument("--c4-microbatches", type=int, default=500)
    ap.add_argument("--streams", type=int, default=3,
                    help="HIP streams (default priority) that the independent passes of a step and the microbatches of the c4 leg "
                         "are spread over, each with its own workspace; 1 = everything on one stream")
    ap.add_argument("--no-sweep", action="store_true",
                    help="leave the size sweep out of the c2 leg (it launches the same kernels on larger tensors, which would "
                         "mix into a profiler's per-kernel averages)")
    args = ap.parse_args()
    if not 1 <= args.streams <= 8:
        print("bench.py: --streams takes 1 to 8", file=sys.stderr)
        return 2
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (tensors shard by microbatch with no exchange); "
              "use --gpus 1", file=sys.stderr)
        return 2
    legs = [l for l in args.legs.split(",") if l]
    for l in legs:
        if l not in ALL_LEGS:
            print(f"bench.py: unknown leg {l!r}", file=sys.stderr)
            return 2

    import torch

    import paper_2211_04515_amd as qp
    import synth_inputs as si

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    qp.lib()
    torch.cuda.set_device(0)
    # The side streams, made once and first.  As measured: the first three streams a process makes overlap fully; streams made
    # after them overlap less (a HIP process has four hardware queues by default, so later streams share one, and two
    # lanes on one queue run one after the other).
    side_streams = [torch.cuda.Stream() for _ in range(args.streams)] if args.streams > 1 else []

    # short kernels (about 10 us): an event pair per launch would add a fifth to them, so kernel_reps
    # back-to-back launches over rotating buffers are timed between two HIP events on the launch stream
    # (a whole untimed repetition first: after a pause on the host the first few milliseconds of GPU work run at a
    # lower clock, which showed as 10-15 % on the first search timed after a synchronising call)
    def timed_reps(fn, reps=None):
        R = reps or args.kernel_reps
        for r in range(R):
            fn(r)
        torch.cuda.synchronize()
        for r in range(R):
            fn(r)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for r in range(R):
            fn(r)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e3 / R

    out = {
        "metric": "activation GB/s quantize+pack & unpack+dequant (% HBM peak); DS-ACIQ us/tensor",
        "value": None, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": None, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
    }
    x_c2 = None
    if "c2" in legs:
        x_c2 = si.make_config("C2")
        out.update(c2_leg(qp, si, torch, x_c2, args, timed_reps, side_streams))
    if "c3" in legs:
        out["c3_vit_large_fp32"] = c3_leg(qp, si, torch, timed_reps, args.kernel_reps)
    if "c5" in legs:
        out["large_tensor_bf16"] = large_tensor_leg(qp, si, torch, timed_reps, args.kernel_reps)
    if "c1" in legs:
        out["small_tensor_fp32"] = small_tensor_leg(qp, si, torch, timed_reps, side_streams)
    if "c4" in legs:
        out["microbatch_stream_fp32"] = c4_stream_leg(qp, si, torch, args.c4_microbatches, side_streams)
    if "cpu" in legs:
        out["cpu_baseline"] = cpu_baseline(x_c2 if x_c2 is not None else si.make_config("C2"), si.CONFIG_BITS["C2"])
    print(json.dumps(out))
    return 0


def c2_leg(qp, si, torch, x_host, args, timed_reps, side_streams):
    """The timed step (whole path, six bitwidths) and the per-kernel rooflines on the ViT-Base tensor."""
    bits_set = si.CONFIG_BITS["C2"]
    n = x_host.size
    in_bytes = n * 4
    xs = [torch.from_numpy(x_host).cuda() for _ in range(NBUF)]
    ys = [torch.empty(n, dtype=torch.float32, device="cuda") for _ in range(NBUF)]
    packs = {b: [qp.alloc_packed(n, b) for _ in range(NBUF)] for b in bits_set}
    ws = qp.alloc_workspace(n)
    qdev = ws.data_ptr() + qp.qp_ws_offset(qp.QP_WS_QPARAMS)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    counter = [0]

    # The six passes of a step are independent jobs (each a whole sender + receiver path at its own bitwidth), so the
    # step hands them round-robin to `--streams` HIP streams of default priority, each with a workspace of its own
    # (qp_compress_many_async): the HBM-bound statistics, pack and unpack of one pass then run beside the
    # vector-ALU-bound search of another.
    lanes = [(s, qp.alloc_workspace(n)) for s in side_streams]

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

    qrecs = torch.zeros(32 * len(bits_set), dtype=torch.uint8, device="cuda")   # the grid record that travels with each payload

    def step_in_flight():
        # sender side: one call, job k on lane k mod len(lanes); receiver side: each payload's unpack behind it on its lane
        ii = [(counter[0] + k) % NBUF for k in range(len(bits_set))]
        counter[0] += len(bits_set)
        qp.qp_compress_many_async([(xs[i], b, packs[b][i], qrecs.data_ptr() + 32 * k) for k, (b, i) in enumerate(zip(bits_set, ii))],
                                  [(w, s) for s, w in lanes])
        for k, (b, i) in enumerate(zip(bits_set, ii)):
            qp.qp_unpack_dequant_dev(packs[b][i], b, qrecs.data_ptr() + 32 * k, ys[i], stream=lanes[k % len(lanes)][0])

    def step(timers=None, overlapped=False):
        if overlapped and lanes:
            return step_in_flight()
        for b in bits_set:
            one_pass(b, timers)

    # four plain device copies of the tensor: under a rocprofv3 counter run these calibrate what
    # FETCH_SIZE / WRITE_SIZE read for a kernel that moves a known number of bytes
    for i in range(4):
        ys[i].copy_(xs[i])
    # Steady-state clock first, whatever --warmup says: after a pause on the host the GPU needs some tens of milliseconds
    # of work to reach the clock it then sustains (timed after 4 ms of work the same steps read 6 % slower).
    t_heat = time.perf_counter() + PREHEAT_S
    while time.perf_counter() < t_heat:
        step(overlapped=True)
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step(overlapped=True)
    torch.cuda.synchronize()
    # timed region: exactly `steps` steps of the fused device-resident path, nothing else on the device
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(overlapped=True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = len(bits_set) * in_bytes / (ms_per_step * 1e-3) / 1e9
    # the same steps with the six passes one after another on one stream (what the stage times below add up to)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step_one_stream = (time.perf_counter() - t0) * 1e3 / args.steps

    # the same `steps` steps again with a HIP event between the stages of every pass (this costs a few
    # microseconds per pass and one extra small launch, so it is kept out of `value`)
    timers = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(timers)
    torch.cuda.synchronize()
    ms_per_step_instrumented = (time.perf_counter() - t0) * 1e3 / args.steps
    stage = {"stats": [], "search": [], "pack": [], "unpack": []}
    for bits, e in timers:
        for k, s in enumerate(("stats", "search", "pack", "unpack")):
            stage[s].append(e[k].elapsed_time(e[k + 1]) * 1e3)
    mean = lambda v: float(sum(v) / len(v))
    search_us = mean(stage["search"])       # setup kernel (a few microseconds) + search kernel
    roofline = alu_entry("k_search_mse<fp32,13> (+ k_search_setup)", n, 101, search_us, TRAFFIC_RATIO["c2_search_bytes"],
                         "HIP events around every search launch in an instrumented repetition of the timed steps")
    roofline["traffic_source"] = TRAFFIC_SOURCE["c2"]

    rot = (f"{args.kernel_reps} back-to-back launches between two HIP events, every stream rotating over at least {NBUF} distinct "
           f"buffers and {COLD_BYTES / 1e6:.0f} MB")
    per_bits = {}
    for b in bits_set:
        q = qp.read_ws(ws, qp.QP_WS_QPARAMS, qp.qp_qparams_t)
        q = qp.qp_make_qparams((q.lo + q.hi) / 2, (q.hi - q.lo) / 2, b, n)
        cold = cold_payloads(qp, torch, xs[0], q, n, b, NBUF)
        tp = timed_reps(lambda r: qp.qp_quant_pack(xs[r % NBUF], q, cold[r % len(cold)]))
        tu = timed_reps(lambda r: qp.qp_unpack_dequant(cold[r % len(cold)], q, ys[r % NBUF]))
        del cold
        byts = in_bytes + n * b / 8
        per_bits[str(b)] = {"pack_us": tp, "pack_GBs": byts / tp / 1e3, "pack_frac_hbm": byts / tp / 1e3 / HBM_PEAK_GBS,
                            "unpack_us": tu, "unpack_GBs": byts / tu / 1e3,
                            "unpack_frac_hbm": byts / tu / 1e3 / HBM_PEAK_GBS}
    ts = timed_reps(lambda r: qp.qp_stats_async(xs[r % NBUF], ws))
    # second reference line beside the nominal 8 TB/s: what a plain device-to-device copy of a tensor of this
    # size reaches under the same timing (one launch per tensor, rotating buffers)
    tcopy = timed_reps(lambda r: ys[r % NBUF].copy_(xs[(r + 1) % NBUF]))
    copy_ref = {"kernel": "torch device-to-device copy (not part of the path)", "bytes": 2 * in_bytes, "us": tcopy,
                "GBs": 2 * in_bytes / tcopy / 1e3}
    # and a write-only one: unpack+dequantize is 80-94 % writes, and a plain fill of its output tensor (torch's fill
    # kernel, same timing and rotation) is the floor for that part
    tfill = timed_reps(lambda r: ys[r % NBUF].fill_(1.5))
    fill_ref = {"kernel": "torch fill of the fp32 output tensor (not part of the path)", "bytes": in_bytes, "us": tfill,
                "GBs": in_bytes / tfill / 1e3}
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
        for k, b in enumerate(bits_set):
            i = (r * len(bits_set) + k) % NBUF          # a different buffer set for every pass, as in the timed step
            qp.qp_compress_async(xs[i], b, ws, packs[b][i], cfg=pol)
            qp.qp_unpack_dequant_dev(packs[b][i], b, qdev, ys[i])
    tpol = timed_reps(policy_step)
    policy = {"ms_per_step": tpol / 1e3, "GBs": len(bits_set) * in_bytes / tpol / 1e3, "streams": 1}
    if lanes:
        def policy_step_in_flight():
            ii = [(counter[0] + k) % NBUF for k in range(len(bits_set))]
            counter[0] += len(bits_set)
            qp.qp_compress_many_async([(xs[i], b, packs[b][i], qrecs.data_ptr() + 32 * k) for k, (b, i) in enumerate(zip(bits_set, ii))],
                                      [(w, s) for s, w in lanes], cfg=pol)
            for k, (b, i) in enumerate(zip(bits_set, ii)):
                qp.qp_unpack_dequant_dev(packs[b][i], b, qrecs.data_ptr() + 32 * k, ys[i], stream=lanes[k % len(lanes)][0])
        for _ in range(args.warmup):
            policy_step_in_flight()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            policy_step_in_flight()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
        policy["in_flight"] = {"ms_per_step": ms, "GBs": len(bits_set) * in_bytes / ms / 1e6, "streams": len(lanes)}

    # Where the floor of a launch of this size is: pack and unpack at 4 bit, and the statistics, on 1, 2, 4 and 8 copies of the tensor
    # laid end to end (38.7 to 310 MB in), each size over enough rotating buffers to exceed the Infinity Cache;
    # least-squares fit of us = fixed + bytes / rate.  The fixed part (launch, ramp to full bandwidth, drain) is what
    # keeps a 40 MB launch below the rate the same kernel reaches on a large tensor.
    sweep = None if args.no_sweep else size_sweep(qp, torch, x_host, timed_reps)

    # headline for pack / unpack: the mean over the six bitwidths of the workload
    pack_bytes = sum(in_bytes + n * b / 8 for b in bits_set)
    pack_us = sum(per_bits[str(b)]["pack_us"] for b in bits_set)
    unpack_us = sum(per_bits[str(b)]["unpack_us"] for b in bits_set)
    nb = len(bits_set)
    r_pack = hbm_entry("k_quant_pack<k,fp32>, k in {2,3,4,6,8,16}", pack_bytes / nb, pack_us / nb, TRAFFIC_RATIO["c2_pack"],
                       TRAFFIC_SOURCE["c2"], rot)
    r_unpack = hbm_entry("k_unpack_dequant<k>, k in {2,3,4,6,8,16}", pack_bytes / nb, unpack_us / nb,
                         TRAFFIC_RATIO["c2_unpack"], TRAFFIC_SOURCE["c2"], rot)
    r_stats = hbm_entry("k_stats_pass1 + k_stats_pass2", 2 * in_bytes, ts, TRAFFIC_RATIO["c2_stats"], TRAFFIC_SOURCE["c2"], rot)
    return {
        "value": value, "ms_per_step": ms_per_step,
        "config": {"workload": "C2 (the configuration the metric is quoted on): ViT-Base stage boundary 64x197x768 fp32, "
                               "70% Laplace(0,0.4)/30% N(0.1,1) + 0.05% outliers x30, full path (stats, DS-ACIQ t=100, pack, "
                               "unpack) once per bitwidth in {2,3,4,6,8,16}; the largest single-GPU configuration (C5, "
                               "256x577x1024 bf16) is the large_tensor_bf16 entry of this line",
                   "elements": n, "bitwidths": list(bits_set), "passes_per_step": nb, "buffers_rotated": NBUF,
                   "streams": max(1, args.streams), "preheat_ms_before_warmup": PREHEAT_S * 1e3},
        "value_is": "activation bytes entering the whole path per second, the six independent passes of a step in flight on "
                    "config.streams streams (one_stream: the same with one pass after the other); the metric's named rates (quantize+pack, "
                    "unpack+dequantize GB/s and % of HBM peak, DS-ACIQ us per tensor) are roofline_pack, roofline_unpack "
                    "and dsaciq_us_per_tensor",
        "one_stream": {"ms_per_step": ms_per_step_one_stream, "GBs": nb * in_bytes / ms_per_step_one_stream / 1e6,
                       "note": "the same steps with the six passes back to back on one stream; stage_us and the rooflines are "
                               "measured this way, so their sum times six is this figure, not ms_per_step"},
        "ms_per_step_instrumented": ms_per_step_instrumented,
        "stage_us": {k: mean(v) for k, v in stage.items()},
        "dsaciq_us_per_tensor": search_us,
        "dsaciq_histogram_fit_us_per_tensor": th,
        "dsaciq_coarse_to_fine_us_per_tensor": tc,
        "step_with_search_at_2_to_4_bit_only": policy,
        "roofline": roofline, "roofline_pack": r_pack, "roofline_unpack": r_unpack, "roofline_stats": r_stats,
        "hbm_copy_reference": copy_ref, "hbm_fill_reference": fill_ref,
        "per_bitwidth": per_bits,
        "size_sweep_4bit": sweep,
    }


def size_sweep(qp, torch, x_host, timed_reps):
    import numpy as np
    n1 = x_host.size
    rows, pts_p, pts_u, pts_s = [], [], [], []
    for m in (1, 2, 4, 8):
        n = n1 * m
        nb = max(3, 16 // m)
        xs = [torch.from_numpy(x_host).cuda().repeat(m) for _ in range(nb)]
        ys = [torch.empty(n, dtype=torch.float32, device="cuda") for _ in range(nb)]
        q = qp.qp_make_qparams(0.0, 2.5, 4, n)
        pk = cold_payloads(qp, torch, xs[0], q, n, 4, nb)
        tp = timed_reps(lambda r: qp.qp_quant_pack(xs[r % nb], q, pk[r % len(pk)]))
        tu = timed_reps(lambda r: qp.qp_unpack_dequant(pk[r % len(pk)], q, ys[r % nb]))
        ws = qp.alloc_workspace(n)
        ts = timed_reps(lambda r: qp.qp_stats_async(xs[r % nb], ws))
        byts = n * 4 + n * 4 / 8
        rows.append({"elements": n, "bytes": byts, "pack_us": tp, "pack_frac_hbm": byts / tp / 1e3 / HBM_PEAK_GBS,
                     "unpack_us": tu, "unpack_frac_hbm": byts / tu / 1e3 / HBM_PEAK_GBS,
                     "stats_bytes": 2 * n * 4, "stats_us": ts, "stats_frac_hbm": 2 * n * 4 / ts / 1e3 / HBM_PEAK_GBS})
        pts_p.append((byts, tp))
        pts_u.append((byts, tu))
        pts_s.append((2 * n * 4, ts))
        del xs, ys, pk, ws

    def fit(pts):
        a = np.array([[1.0, b] for b, _ in pts])
        t = np.array([u for _, u in pts])
        (fixed, slope), *_ = np.linalg.lstsq(a, t, rcond=None)
        return {"fixed_us": float(fixed), "asymptotic_GBs": float(1.0 / slope / 1e3),
                "asymptotic_frac_hbm": float(1.0 / slope / 1e3 / HBM_PEAK_GBS)}
    return {"sizes": rows, "fit_pack": fit(pts_p), "fit_unpack": fit(pts_u), "fit_stats_two_launches": fit(pts_s)}


def c3_leg(qp, si, torch, timed_reps, reps):
    """C3: the ViT-Large stage boundary 64x197x1024 fp32 after a GELU (one-sided, spike near zero), searched with
    cands_per_round = 32 as the configuration names it (an upper bound to the library, which takes rounds of 13 / 12
    candidates: more per round leaves too few waves per SIMD), bitwidths {2,4,8}."""
    x = si.make_config("C3")
    n = x.size
    in_bytes = n * 4
    nb = 12                                       # 620 MB of inputs in rotation
    xs = [torch.from_numpy(x).cuda() for _ in range(nb)]
    ys = [torch.empty(n, dtype=torch.float32, device="cuda") for _ in range(nb)]
    cfg = qp.qp_default_search_cfg()
    cfg.cands_per_round = 32
    ws = qp.alloc_workspace(n, cfg)
    st = qp.qp_stats(xs[0], ws)
    rot = (f"{reps} back-to-back launches between two HIP events, every stream rotating over at least {nb} distinct buffers "
           f"and {COLD_BYTES / 1e6:.0f} MB")
    ts = timed_reps(lambda r: qp.qp_stats_async(xs[r % nb], ws))
    out = {"elements": n, "input": "fp32", "cands_per_round": 32, "buffers_rotated": nb,
           "roofline_stats": hbm_entry("k_stats_pass1 + k_stats_pass2", 2 * in_bytes, ts, None, None, rot), "per_bitwidth": {}}
    for b in si.CONFIG_BITS["C3"]:
        res, q = qp.qp_dsaciq_search(xs[0], st, b, ws, cfg=cfg)
        packs = cold_payloads(qp, torch, xs[0], q, n, b, nb)
        tsr = timed_reps(lambda r: qp.qp_dsaciq_search_async(xs[r % nb], b, ws, cfg=cfg), 24)
        tp = timed_reps(lambda r: qp.qp_quant_pack(xs[r % nb], q, packs[r % len(packs)]))
        tu = timed_reps(lambda r: qp.qp_unpack_dequant(packs[r % len(packs)], q, ys[r % nb]))
        tsend = timed_reps(lambda r: qp.qp_compress_async(xs[r % nb], b, ws, packs[r % len(packs)], cfg=cfg), 24)
        byts = in_bytes + n * b / 8
        out["per_bitwidth"][str(b)] = {
            "j_star": res.j_star, "mse_star_over_mse_aciq": res.mse_star / res.mse_aciq,
            "sender_path_us_per_tensor": tsend,
            "roofline_search": alu_entry("k_search_mse<fp32,13> (+ k_search_setup)", n, 101, tsr, None,
                                         "24 back-to-back searches over rotating inputs between two HIP events"),
            "roofline_pack": hbm_entry(f"k_quant_pack<{b},fp32>", byts, tp, None, None, rot),
            "roofline_unpack": hbm_entry(f"k_unpack_dequant<{b}>", byts, tu, None, None, rot)}
        del packs
    return out


def large_tensor_leg(qp, si, torch, timed_reps, reps):
    """C5: statistics, search, quantize+pack and unpack+dequantize on the 256x577x1024 bf16 tensor (Student-t, df 3,
    x0.5): 302 MB in, larger than the Infinity Cache by itself, so every launch is served by HBM."""
    h = si.make_config("C5")
    n = h.size
    nb = 3
    xs = [torch.from_numpy(h.view("int16").copy()).cuda().view(torch.bfloat16) for _ in range(nb)]
    ys = [torch.empty(n, dtype=torch.float32, device="cuda") for _ in range(nb)]
    ws = qp.alloc_workspace(n)
    # plain device copies of known size: the calibration of FETCH_SIZE / WRITE_SIZE under a counter run
    for i in range(nb):
        ys[(i + 1) % nb].copy_(ys[i])
    st = qp.qp_stats(xs[0], ws)
    rot = (f"{reps} back-to-back launches between two HIP events, every stream rotating over at least {nb} distinct buffers "
           f"and {COLD_BYTES / 1e6:.0f} MB")
    t_stats = timed_reps(lambda r: qp.qp_stats_async(xs[r % nb], ws))
    out = {"elements": n, "input": "bf16", "buffers_rotated": nb, "stats_us": t_stats,
           # a bf16 tensor of this size goes through its value table: ONE read of the tensor (2 B per element) instead of
           # the two passes (4 B per element) the two-pass statistics need; the rate is quoted on the one read
           "roofline_stats": hbm_entry("k_value_table_zero + k_value_hist_bf16 + k_stats_from_table (one read of the tensor)",
                                       n * 2, t_stats, TRAFFIC_RATIO["c5_value_hist"], TRAFFIC_SOURCE["c5"], rot)}
    tcopy = timed_reps(lambda r: ys[(r + 1) % nb].copy_(ys[r % nb]))
    out["hbm_copy_reference_GBs"] = 2 * n * 4 / tcopy / 1e3   # plain device-to-device copy of the fp32 output tensor
    tfill = timed_reps(lambda r: ys[r % nb].fill_(1.5))
    out["hbm_fill_reference_GBs"] = n * 4 / tfill / 1e3       # plain fill of it: the write-only floor of unpack+dequantize
    out["per_bitwidth"] = {}
    for b in si.CONFIG_BITS["C5"]:
        res, q = qp.qp_dsaciq_search(xs[0], st, b, ws)
        packs = cold_payloads(qp, torch, xs[0], q, n, b, nb)
        tp = timed_reps(lambda r: qp.qp_quant_pack(xs[r % nb], q, packs[r % len(packs)]))
        tu = timed_reps(lambda r: qp.qp_unpack_dequant(packs[r % len(packs)], q, ys[r % nb]))
        ts = timed_reps(lambda r: qp.qp_dsaciq_search_async(xs[r % nb], b, ws))
        tsend = timed_reps(lambda r: qp.qp_compress_async(xs[r % nb], b, ws, packs[r % len(packs)]))
        bp, bu = n * 2 + n * b / 8, n * 4 + n * b / 8
        out["per_bitwidth"][str(b)] = {
            "j_star": res.j_star,
            # search alone = table zero + value-count pass over the tensor + 101 candidates over the 65536-entry table
            "dsaciq_us_per_tensor": ts, "sender_path_us_per_tensor": tsend,
            "roofline_pack": hbm_entry(f"k_quant_pack<{b},bf16>", bp, tp, TRAFFIC_RATIO["c5_pack"], TRAFFIC_SOURCE["c5"], rot),
            "roofline_unpack": hbm_entry(f"k_unpack_dequant<{b}>", bu, tu, TRAFFIC_RATIO["c5_unpack"], TRAFFIC_SOURCE["c5"], rot)}
        del packs
    return out


def c4_stream_leg(qp, si, torch, n_mb, side_streams):
    """C4: sender path + receiver per microbatch (32x257x1280 fp32, 42 MB) over a ring of eight unit-Laplace buffers
    scaled per microbatch on the device; the bitwidth of each microbatch follows the seeded bandwidth trace.  All n_mb
    inputs (21 GB at 500) are resident before the timed region.  Timed twice: back to back on one stream, and with the
    microbatches handed round-robin to the side streams (a workspace, payload and output buffer each)."""
    n = si.numel("C4")
    stream = si.c4_stream(n_mb)
    ring = [torch.from_numpy(si.unit_laplace(n, 100 + b)).cuda() for b in range(8)]
    xs = [ring[buf] * b_m for (buf, b_m, bw, bits) in stream]          # n_mb x 42 MB, all distinct
    kset = sorted({s[3] for s in stream})
    lanes = [(s, qp.alloc_workspace(n), {k: qp.alloc_packed(n, k) for k in kset}, torch.empty(n, dtype=torch.float32, device="cuda"))
             for s in (side_streams or [None])]

    def run(nl):
        for m, (x, (_, _, _, bits)) in enumerate(zip(xs, stream)):
            s, ws, packs, y = lanes[m % nl]
            s = s if nl > 1 else None
            qp.qp_compress_async(x, bits, ws, packs[bits], stream=s)
            qp.qp_unpack_dequant_dev(packs[bits], bits, ws.data_ptr() + qp.qp_ws_offset(qp.QP_WS_QPARAMS), y, stream=s)

    def timed(nl):
        run(nl)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run(nl)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e6 / n_mb

    us_one = timed(1)
    us = timed(len(lanes)) if len(lanes) > 1 else us_one
    hist = {}
    for s_ in stream:
        hist[str(s_[3])] = hist.get(str(s_[3]), 0) + 1
    return {"elements_per_microbatch": n, "microbatches": n_mb, "input_bytes_resident": n_mb * n * 4,
            "bitwidths_used": hist, "streams": len(lanes), "us_per_microbatch": us, "activation_GBs": n * 4 / us / 1e3,
            "one_stream": {"us_per_microbatch": us_one, "activation_GBs": n * 4 / us_one / 1e3},
            "timed": "statistics, DS-ACIQ (t = 100), quantize+pack, unpack+dequantize per microbatch; host clock around all "
                     "microbatches between two device synchronisations"}


def small_tensor_leg(qp, si, torch, timed_reps, side_streams):
    """C1: sender path (statistics, DS-ACIQ t = 100, quantize+pack) and its search alone on the 1x197x768 tensor,
    launched eagerly and replayed from a HIP graph that holds 16 sender paths over rotating inputs."""
    x = si.make_config("C1")
    n = x.size
    nb = 4
    xs = [torch.from_numpy(x).cuda() for _ in range(nb)]
    ws = qp.alloc_workspace(n)
    packed = qp.alloc_packed(n, 4)
    qp.qp_stats(xs[0], ws)
    t_search = timed_reps(lambda r: qp.qp_dsaciq_search_async(xs[r % nb], 4, ws))
    t_send = timed_reps(lambda r: qp.qp_compress_async(xs[r % nb], 4, ws, packed))
    # the same 16 sender paths captured once and replayed: what the launch overhead of the five kernels costs
    per_graph = 16
    s = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        for r in range(per_graph):
            qp.qp_compress_async(xs[r % nb], 4, ws, packed)
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=s):
        for r in range(per_graph):
            qp.qp_compress_async(xs[r % nb], 4, ws, packed)
    torch.cuda.synchronize()
    t_graph = timed_reps(lambda r: g.replay(), 16) / per_graph
    out = {"elements": n, "bits": 4, "dsaciq_us_per_tensor": t_search, "sender_path_us_per_tensor": t_send,
           "sender_path_us_per_tensor_graph_replay": t_graph,
           "timed": "back-to-back calls on one stream between two HIP events; graph: 16 replays of a HIP graph holding 16 sender paths"}
    if side_streams:
        # independent tensors in flight: the same sender paths handed round-robin to the side streams (a workspace and a
        # payload buffer each); host clock around 3 x 256 tensors between two device synchronisations, best of three
        lanes = [(st, qp.alloc_workspace(n), qp.alloc_packed(n, 4)) for st in side_streams]
        per = 256

        def burst():
            for r in range(per):
                st, w, pk = lanes[r % len(lanes)]
                qp.qp_compress_async(xs[r % nb], 4, w, pk, stream=st)
        burst()
        torch.cuda.synchronize()
        best = None
        for _ in range(3):
            t0 = time.perf_counter()
            burst()
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) * 1e6 / per
            best = dt if best is None else min(best, dt)
        out["sender_path_us_per_tensor_in_flight_on_side_streams"] = {"streams": len(lanes), "us_per_tensor": best}
        # the same with one HIP graph of 16 sender paths per side stream, replayed side by side (the eager burst above is
        # bound by the host's launch rate: five launches per tensor)
        graphs = []
        for st, w, pk in lanes:
            gk = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gk, stream=st):
                for r in range(per_graph):
                    qp.qp_compress_async(xs[r % nb], 4, w, pk)
            graphs.append((st, gk))
        torch.cuda.synchronize()

        def replay_all(rounds):
            for _ in range(rounds):
                for st, gk in graphs:
                    with torch.cuda.stream(st):
                        gk.replay()
        replay_all(4)
        torch.cuda.synchronize()
        best = None
        for _ in range(3):
            t0 = time.perf_counter()
            replay_all(16)
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) * 1e6 / (16 * len(graphs) * per_graph)
            best = dt if best is None else min(best, dt)
        out["sender_path_us_per_tensor_in_flight_graph_replay"] = {"streams": len(lanes), "us_per_tensor": best}
    return out


def cpu_baseline(x_host, bits_set):
    """The oracle as it stands (never tuned) on the first quarter of the C2 tensor, all six bitwidths: once on a
    single thread, and once with the timing harness spreading the same calls over the host's cores (the search's
    candidates over threads; statistics, quantize, pack, unpack and dequantize over contiguous chunks of the tensor
    whose lengths are multiples of 32 codes).  The oracle's code is the same in both."""
    from concurrent.futures import ThreadPoolExecutor

    from oracle import qp_oracle as orc
    sample = x_host[: x_host.size // 4]
    n = sample.size
    t0 = time.perf_counter()
    rc, st = orc.stats(sample)
    for b in bits_set:
        res, q, _ = orc.dsaciq_search(sample, st, b, 100)
        codes = orc.quantize(sample, q)
        stream = orc.pack(codes, b)
        y = orc.dequantize(orc.unpack(stream, n, b), q)
    dt1 = time.perf_counter() - t0

    ncpu = os.cpu_count() or 1
    try:
        ncpu = min(ncpu, len(os.sched_getaffinity(0)))
    except (AttributeError, OSError):
        pass
    threads = max(1, min(16, ncpu))           # the share of a one-GPU machine
    step = ((n + threads - 1) // threads + 31) // 32 * 32
    chunks = [sample[i:i + step] for i in range(0, n, step)]
    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=threads) as ex:
        list(ex.map(orc.stats, chunks))                                  # timing only: per-chunk statistics
        for b in bits_set:
            res, q, _ = orc.dsaciq_search_threads(sample, st, b, 100, threads)
            list(ex.map(lambda c: orc.dequantize(orc.unpack(orc.pack(orc.quantize(c, q), b), c.size, b), q), chunks))
    dtn = time.perf_counter() - t0
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    work = len(bits_set) * n * 4
    return {"value": work / dt1 / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"first quarter of the C2 tensor ({n} elements), all six bitwidths, {dt1:.1f} s of CPU time",
            "seconds": dt1,
            "all_cores": {"value": work / dtn / 1e9, "unit": "GB/s", "cores": threads, "seconds": dtn,
                          "how": "same oracle calls; the timing harness spreads the search's candidates and contiguous "
                                 "chunks of the tensor over host threads"},
            "host": {"cpu_model": model, "os_cpu_count": os.cpu_count(), "usable_cpus": ncpu}}


if __name__ == "__main__":
    sys.exit(main())
