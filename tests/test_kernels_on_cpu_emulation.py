"""The library's kernel sources, compiled by the host compiler against a CPU stand-in for the HIP runtime
(tests/emu/) and run under AddressSanitizer + UBSan on tiny tensors, against the oracle.

What this adds to the GPU parity tests: it runs without a GPU, and the sanitizers see every access of every
kernel against buffers of exactly the sizes the C ABI asks for (workspace, packed stream), so an index
that strays fails here first.  By default the blocks of a launch run one after the other in index order; the
"concurrent" cases run them several at a time in a shuffled order, each block in a process of its own over
shared "device memory", so that the ticket hand-overs between blocks (last block of a round, last round of a
search, last block of the statistics) are taken in many orders.  What it cannot show: speed, and the device's
memory model (the host orders stores more strongly than the GPU's caches do).  The emulation is test
infrastructure; the library has no CPU path."""
import ctypes as C
import os
import subprocess
import sys

import numpy as np
import pytest

import synth_inputs as si
from oracle import qp_oracle as orc

sys.path.insert(0, os.path.join(os.path.dirname(os.path.abspath(__file__)), "emu"))
import build_emu  # noqa: E402

REL = 1e-11


class Stats(C.Structure):
    _fields_ = [("n", C.c_uint64), ("n_nonfinite", C.c_uint64), ("mean", C.c_double), ("mad", C.c_double),
                ("abs_mean", C.c_double), ("var", C.c_double), ("min", C.c_double), ("max", C.c_double),
                ("nbins", C.c_uint32), ("peak_count", C.c_uint32), ("peak_density", C.c_double), ("b_r", C.c_double)]


class QParams(C.Structure):
    _fields_ = [("bits", C.c_uint32), ("reserved", C.c_uint32), ("n", C.c_uint64), ("lo", C.c_float), ("hi", C.c_float),
                ("scale", C.c_float), ("inv_scale", C.c_float)]


class Result(C.Structure):
    _fields_ = [("b_e", C.c_double), ("b_r", C.c_double), ("b_star", C.c_double), ("alpha_star", C.c_double),
                ("mse_aciq", C.c_double), ("mse_star", C.c_double), ("j_star", C.c_uint32), ("t_steps", C.c_uint32)]


@pytest.fixture(scope="module")
def drivers():
    try:
        out = build_emu.build_all()
    except subprocess.CalledProcessError as e:
        pytest.fail("emulation build failed:\n" + e.stderr.decode()[-3000:])
    if any(v is None for v in out.values()):
        pytest.skip("no host clang++ to build the emulation with")
    return out


def start_driver(exe, out_dir, x, bits, t=100, dist=0, flags=0, stride=0, nbins=2048, cus=4, cpr=None, concurrent=0, seed=1):
    os.makedirs(out_dir, exist_ok=True)
    inp = os.path.join(out_dir, "in.bin")
    x.tofile(inp)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    if concurrent:
        env.update(EMU_CONCURRENT_BLOCKS=str(concurrent), EMU_SEED=str(seed))
    return subprocess.run([exe, inp, str(x.size), "1" if x.dtype == np.uint16 else "0", str(bits), str(t), str(dist),
                           str(flags), str(stride), str(nbins), str(cus), out_dir] + ([str(cpr)] if cpr else []),
                          capture_output=True, env=env, timeout=900)


def read_outputs(p, out_dir):
    assert p.returncode == 0, "sanitizer report or crash:\n" + p.stderr.decode()[-4000:]
    path = lambda name: os.path.join(out_dir, name)
    rc = [int(v) for v in open(path("status.txt")).read().split()]
    rd = lambda name, dt: np.fromfile(path(name), dtype=dt)
    return dict(rc=rc, stats=Stats.from_buffer_copy(open(path("stats.bin"), "rb").read()),
                res=Result.from_buffer_copy(open(path("result.bin"), "rb").read()),
                q=QParams.from_buffer_copy(open(path("qparams.bin"), "rb").read()),
                hist=rd("hist.bin", np.uint32), scores=rd("scores.bin", np.float64), packed=rd("packed.bin", np.uint8),
                scores2=rd("scores2.bin", np.float64), res2=Result.from_buffer_copy(open(path("result2.bin"), "rb").read()),
                y=rd("y.bin", np.float32))


def check_against_oracle(r, x, bits, t=100, dist=0, clip=False, stride=1, nbins=2048):
    xf = orc.widen_bf16(x) if x.dtype == np.uint16 else x
    n = x.size
    assert r["rc"] == [0, 0, 0, 0, 0, 1]        # every call succeeded; the fused sender path equals the step-by-step calls
    st = r["stats"]
    rc, ref, hist_ref = orc.stats(xf, nbins=nbins, want_hist=True)
    assert (st.n, st.n_nonfinite, st.min, st.max, st.nbins, st.peak_count) == (n, 0, ref.min, ref.max, nbins, ref.peak_count)
    for f in ("mean", "mad", "abs_mean", "var"):
        a, b = getattr(st, f), getattr(ref, f)
        assert abs(a - b) <= REL * max(abs(b), ref.abs_mean * 1e-3 if f == "mean" else 0.0), f
    assert np.array_equal(r["hist"], hist_ref[:nbins])
    ost = orc.Stats()
    for name, _ in orc.Stats._fields_:
        setattr(ost, name, getattr(st, name))
    if dist == 2:   # the model chosen on the (emulated) device by fit: the oracle makes the same choice from the same record
        dist = orc.model_fit(ost, r["hist"])[0]
    ores, oq, oscores = orc.dsaciq_search_variant(xf, ost, bits, t, dist=dist, clip_to_data=clip, stride=stride)
    assert np.array_equal(np.isnan(r["scores"]), np.isnan(oscores))
    assert np.allclose(r["scores"], oscores, rtol=REL, atol=0.0, equal_nan=True)
    # the fused sender path's own search (for small tensors: the pick folded into the search kernel)
    assert np.array_equal(np.isnan(r["scores2"]), np.isnan(oscores))
    assert np.allclose(r["scores2"], oscores, rtol=REL, atol=0.0, equal_nan=True)
    assert (r["res2"].j_star, r["res2"].t_steps) == (ores.j_star, t)
    assert r["res2"].mse_star == pytest.approx(ores.mse_star, rel=REL, nan_ok=True) and r["res2"].mse_aciq == pytest.approx(ores.mse_aciq, rel=REL, nan_ok=True)
    res, q = r["res"], r["q"]
    assert res.j_star == ores.j_star and res.t_steps == t
    assert res.alpha_star == pytest.approx(ores.alpha_star, rel=1e-14)
    assert (q.bits, q.n, q.lo, q.hi, q.scale, q.inv_scale) == (bits, n, oq.lo, oq.hi, oq.scale, oq.inv_scale)
    codes = orc.quantize(xf, oq)
    assert np.array_equal(r["packed"], orc.pack(codes, bits))
    assert np.array_equal(r["y"], orc.dequantize(codes, oq))


def small_input(kind, n):
    if kind == "bf16":
        return si.make_config("C5", n=n)
    if kind == "gauss":
        return (np.random.default_rng(n).standard_normal(n) * 0.8 + 0.3).astype(np.float32)
    if kind == "gauss_bf16":
        return si.f32_to_bf16_bits((np.random.default_rng(n).standard_normal(n) * 0.8 + 0.3).astype(np.float32))
    return si.make_config(kind, n=n)


# (kind, n, bits, variant, t): one case sweeps the paper's t = 100, the others a shorter grid (one emulated block
# per candidate in the pick kernel makes t the main cost here)
TILE_CASES = [("C1", 3_011, 2, {}, 100), ("C3", 4_999, 3, {}, 12), ("bf16", 5_345, 4, {}, 12), ("C2", 4_097, 16, {}, 7),
              ("C3", 130, 6, {}, 12), ("C3", 3_001, 4, dict(clip=True), 12), ("C2", 2_191, 2, dict(dist=1, stride=4), 20),
              ("bf16", 2_777, 8, dict(stride=3, clip=True), 12), ("C1", 5, 4, {}, 5), ("C3", 1, 8, {}, 3),
              # the model chosen per tensor by fit (Gaussian data must take the Gaussian model, Laplace-like data the paper's)
              ("gauss", 4_001, 4, dict(dist=2), 12), ("C1", 3_011, 3, dict(dist=2, clip=True), 12), ("gauss", 2_500, 2, dict(dist=2, stride=4), 20)]
# the same kind of tensors through the kernels large tensors take (thresholds lowered at build time)
STREAM_CASES = [("C3", 10_011, 2, {}, 100), ("C2", 6_007, 8, dict(clip=True), 37), ("bf16", 5_001, 4, {}, 30),
                ("bf16", 3_000, 3, dict(dist=1), 20), ("C1", 2_049, 6, {}, 1),
                # the search over the value table with the Gaussian model and ranges intersected with the data's
                ("bf16", 4_500, 3, dict(dist=1, clip=True), 20),
                # rounds of 1, 2, 4 and 3 candidates (cands_per_round 1, 2, 5 with 9 candidates: 4 + 3 + 2 does not split,
                # 3 + 3 + 3 does)
                ("C3", 4_111, 4, dict(cpr=1), 5), ("C2", 4_100, 3, dict(cpr=2), 6), ("C4", 4_321, 2, dict(cpr=5), 8),
                # a coarse-to-fine sweep of a tensor above the tile search's size limit still runs on the tile search
                ("C3", 9_001, 4, dict(stride=5), 40),
                # the model chosen by fit, through the streaming search and through the value table
                ("gauss", 6_001, 4, dict(dist=2), 20), ("gauss_bf16", 5_003, 3, dict(dist=2), 20), ("C2", 5_555, 2, dict(dist=2, cpr=4), 9)]
REFUSED = ("bf16", 5_000, 4, dict(stride=10), 100)
ACIQ_ONLY = [("default", ("C3", 3_003, 8, dict(low_bits_only=True), 100)), ("streaming", ("bf16", 6_001, 6, dict(low_bits_only=True, clip=True), 100))]
# Blocks of a launch in shuffled order, `conc` at a time (each a process of its own): ticket hand-overs out of order.
# The tile search and its pick kernel, the streaming search with several rounds, the statistics finalizer, the
# value-table search; two seeds each.
CONCURRENT_CASES = [("default", ("C2", 9_001, 4, dict(conc=3, seed=1), 12)), ("default", ("C2", 9_001, 4, dict(conc=3, seed=2), 12)),
                    ("streaming", ("C3", 10_011, 2, dict(conc=4, seed=1), 30)), ("streaming", ("C3", 10_011, 2, dict(conc=4, seed=2), 30)),
                    ("streaming", ("C2", 6_007, 8, dict(conc=2, seed=3, cpr=4), 17)),
                    ("streaming", ("bf16", 5_001, 4, dict(conc=4, seed=1), 20)), ("streaming", ("bf16", 5_001, 4, dict(conc=3, seed=2), 20))]
# The sequence the library refuses (a coarse-to-fine search as two sweeps of the STREAMING kernel, the run that once
# faulted a GPU), on the build that allows it: in block order, and with blocks shuffled and concurrent.  One-round
# lists (11 / 19 candidates under 13 per round) and lists of several rounds (cands_per_round 4).
STREAM_C2F_CASES = [("streaming_c2f", ("C3", 10_011, 2, dict(stride=10), 100)),
                    ("streaming_c2f", ("C3", 10_011, 2, dict(stride=10, conc=4, seed=1), 100)),
                    ("streaming_c2f", ("C3", 10_011, 2, dict(stride=10, conc=4, seed=2), 100)),
                    ("streaming_c2f", ("C3", 10_011, 4, dict(stride=10, conc=3, seed=3, cpr=4), 100)),
                    ("streaming_c2f", ("C2", 8_193, 3, dict(stride=5, clip=True, conc=2, seed=4), 40)),
                    ("streaming_c2f", ("C3", 6_007, 4, dict(stride=64, conc=4, seed=5), 100))]
ALL_CASES = ([("default", c) for c in TILE_CASES] + [("streaming", c) for c in STREAM_CASES] + [("streaming", REFUSED)] + ACIQ_ONLY
             + CONCURRENT_CASES + STREAM_C2F_CASES)


def case_id(tag, c):
    return f"{tag}-{c[0]}_{c[1]}_k{c[2]}_t{c[4]}" + "".join(f"_{k}{v}" for k, v in sorted(c[3].items()))


@pytest.fixture(scope="module")
def runs(drivers, tmp_path_factory):
    """Every case's driver run, started together (each run is one process with a thread per emulated lane)."""
    from concurrent.futures import ThreadPoolExecutor
    base = str(tmp_path_factory.mktemp("emu"))

    def go(item):
        tag, (kind, n, bits, v, t) = item
        x = small_input(kind, n)
        flags = (1 if v.get("clip") else 0) | (2 if v.get("stride", 1) > 1 else 0) | (4 if v.get("low_bits_only") else 0)
        out_dir = os.path.join(base, case_id(tag, item[1]))
        p = start_driver(drivers[tag], out_dir, x, bits, t=t, dist=v.get("dist", 0), flags=flags,
                         stride=v.get("stride", 0) if flags & 2 else 0, cus=4 if tag == "default" else 2, cpr=v.get("cpr"),
                         concurrent=v.get("conc", 0), seed=v.get("seed", 1))
        return case_id(tag, item[1]), (p, out_dir, x)

    with ThreadPoolExecutor(max_workers=6) as ex:
        return dict(ex.map(go, ALL_CASES))


WHOLE = [a for a in ALL_CASES if a[1] is not REFUSED and a not in ACIQ_ONLY]


@pytest.mark.parametrize("tag,case", WHOLE, ids=[case_id(*a) for a in WHOLE])
def test_whole_path_on_the_emulation(runs, tag, case):
    """Statistics, search (tile search with the default thresholds; streaming search with rounds and tickets and,
    for bf16 of at least 4096 elements, the value table with the lowered ones), quantize+pack, unpack+dequantize
    and the fused sender path: sanitizer-clean and equal to the oracle."""
    kind, n, bits, v, t = case
    p, out_dir, x = runs[case_id(tag, case)]
    r = read_outputs(p, out_dir)
    check_against_oracle(r, x, bits, t=t, dist=v.get("dist", 0), clip=bool(v.get("clip")), stride=v.get("stride", 1))


def test_emulation_refuses_what_the_library_refuses(runs):
    """Coarse-to-fine is not offered for bf16 tensors that go through their value table: QP_EINVAL, nothing more runs."""
    p, out_dir, x = runs[case_id("streaming", REFUSED)]
    r = read_outputs(p, out_dir)
    assert r["rc"][0] == 0 and r["rc"][1] == -1


@pytest.mark.parametrize("tag,case", ACIQ_ONLY, ids=[case_id(*a) for a in ACIQ_ONLY])
def test_low_bits_only_policy_on_the_emulation(runs, tag, case):
    """Above 4 bit with QP_SEARCH_LOW_BITS_ONLY nothing is scored: the result is plain ACIQ from the statistics."""
    kind, n, bits, v, t = case
    p, out_dir, x = runs[case_id(tag, case)]
    r = read_outputs(p, out_dir)
    xf = orc.widen_bf16(x) if x.dtype == np.uint16 else x
    assert r["rc"] == [0, 0, 0, 0, 0, 1]
    st, res, q = r["stats"], r["res"], r["q"]
    ost = orc.Stats()
    for name, _ in orc.Stats._fields_:
        setattr(ost, name, getattr(st, name))
    alpha = orc.aciq_alpha(ost, bits)
    oq = orc.make_qparams_clipped(st.mean, alpha, st.min, st.max, bits, n) if v.get("clip") else orc.make_qparams(st.mean, alpha, bits, n)
    assert res.j_star == 0 and np.isnan(r["scores"]).all() and np.isnan(res.mse_star)
    assert res.alpha_star == pytest.approx(alpha, rel=1e-15)
    assert (q.bits, q.n, q.lo, q.hi, q.scale, q.inv_scale) == (bits, n, oq.lo, oq.hi, oq.scale, oq.inv_scale)
    codes = orc.quantize(xf, oq)
    assert np.array_equal(r["packed"], orc.pack(codes, bits)) and np.array_equal(r["y"], orc.dequantize(codes, oq))
