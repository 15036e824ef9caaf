"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares,
rejects bad arguments before touching the GPU, and its host-only functions agree with the
oracle.  No kernel is launched here."""
import ctypes as C
import math
import os
import re

import numpy as np
import pytest
import scipy.special

from oracle import qp_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BITS = (2, 3, 4, 6, 8, 16)


@pytest.fixture(scope="module")
def qp():
    import paper_2211_04515_amd as m
    m.lib()
    return m


def declared_functions():
    text = open(os.path.join(ROOT, "include", "quantpipe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qp_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(qp):
    names = declared_functions()
    assert len(names) >= 17 and "qp_stats" in names and "qp_unpack_dequant" in names
    raw = C.CDLL(os.path.join(ROOT, "paper_2211_04515_amd", "libquantpipe.so"))
    for n in names:
        assert hasattr(raw, n), f"{n} declared in quantpipe.h but not exported"
    from paper_2211_04515_amd import binding
    assert sorted(binding.EXPORTS) == names          # the Python binding wraps all of them, same names
    for n in names:
        assert callable(getattr(qp, n))


def test_no_alloc_entry_point_refuses_before_touching_the_gpu(qp):
    """Sizes beyond the static workspace and bad arguments are refused by checks that precede every HIP call."""
    L, fake, big = qp.lib(), C.c_void_p(0x10000), 1 << 40
    cfg = qp.qp_default_search_cfg()
    cfg.t_steps = 128
    assert L.qp_compress_noalloc(fake, 1000, 0, 4, C.byref(cfg), fake, big, fake, None) == qp.QP_ENOSPC
    cfg.t_steps = 0
    assert L.qp_compress_noalloc(fake, 1000, 0, 4, C.byref(cfg), fake, big, fake, None) == qp.QP_EINVAL
    assert L.qp_compress_noalloc(fake, 0, 0, 4, None, fake, big, fake, None) == qp.QP_EINVAL
    assert L.qp_compress_noalloc(fake, 2 ** 32, 0, 4, None, fake, big, fake, None) == qp.QP_EINVAL
    assert L.qp_compress_noalloc(fake, 1000, 0, 4, None, fake, big, None, None) == qp.QP_EINVAL


def test_many_tensor_entry_point_checks_every_job_before_touching_the_gpu(qp):
    """Bad lanes, overlapping workspaces and a bad job anywhere in the list are refused by checks that precede every HIP
    call (the pointers here are not device memory: a launch would fail differently)."""
    L = qp.lib()
    need = qp.qp_workspace_bytes(1000)
    pk = qp.qp_packed_bytes(1000, 4)
    assert C.sizeof(qp.qp_job_t) == 48 and C.sizeof(qp.qp_lane_t) == 24

    def job(x=0x10000, n=1000, dtype=0, bits=4, packed=0x20000, packed_bytes=pk, q=0x30000):
        return qp.qp_job_t(x, n, dtype, bits, packed, packed_bytes, q)

    def call(jobs, lanes, count=None, n_lanes=None):
        ja = (qp.qp_job_t * max(1, len(jobs)))(*jobs)
        la = (qp.qp_lane_t * max(1, len(lanes)))(*lanes)
        return L.qp_compress_many_async(ja, len(jobs) if count is None else count, None, la,
                                        len(lanes) if n_lanes is None else n_lanes)

    two = [qp.qp_lane_t(0x100000, need, None), qp.qp_lane_t(0x100000 + need, need, None)]
    good = [job(), job(), job()]
    assert L.qp_compress_many_async(None, 1, None, (qp.qp_lane_t * 2)(*two), 2) == qp.QP_EINVAL
    assert L.qp_compress_many_async((qp.qp_job_t * 3)(*good), 3, None, None, 2) == qp.QP_EINVAL
    assert call(good, two, count=0) == qp.QP_EINVAL
    assert call(good, two, n_lanes=0) == qp.QP_EINVAL
    assert call(good, two * 40) == qp.QP_EINVAL                                        # more than 64 lanes
    assert call(good, [two[0], qp.qp_lane_t(0x100000 + need - 16, need, None)]) == qp.QP_EINVAL   # workspaces overlap
    assert call(good, [two[0], qp.qp_lane_t(None, need, None)]) == qp.QP_EINVAL
    assert call(good, [two[0], qp.qp_lane_t(0x100000 + need, need - 16, None)]) == qp.QP_ENOSPC   # lane 1 too small for job 1
    assert call([job(), job(), job(bits=5)], two) == qp.QP_EINVAL                      # the last job is bad: nothing ran
    assert call([job(), job(dtype=7), job()], two) == qp.QP_EINVAL
    assert call([job(), job(packed_bytes=pk - 4), job()], two) == qp.QP_ENOSPC
    assert call([job(x=0x10004), job(), job()], two) == qp.QP_EINVAL                   # misaligned tensor
    # job 0's lane is reused by job 2, so job 0 needs a place for its grid; jobs 1 and 2 are the last of their lanes
    assert call([job(q=None), job(), job()], two) == qp.QP_EINVAL


def test_struct_sizes_match_the_header_layout(qp):
    assert C.sizeof(qp.qp_stats_t) == 88
    assert C.sizeof(qp.qp_qparams_t) == 32
    assert C.sizeof(qp.qp_search_cfg_t) == 24
    assert C.sizeof(qp.qp_search_result_t) == 56
    offs = [qp.qp_ws_offset(r) for r in range(6)]
    assert offs == sorted(offs) and len(set(offs)) == 6 and all(o % 16 == 0 for o in offs)
    assert qp.qp_ws_offset(99) == 2 ** 64 - 1
    assert C.sizeof(qp.qp_model_fit_t) == 24
    m = qp.qp_ws_offset(qp.QP_WS_MODEL)     # sits in the gap between the winner's grid and the control block
    assert m % 8 == 0 and qp.qp_ws_offset(qp.QP_WS_QPARAMS) + 32 <= m and m + 24 <= qp.qp_ws_offset(qp.QP_WS_HIST)


def test_packed_bytes(qp):
    for bits in BITS:
        for n in (0, 1, 31, 32, 33, 1000, 9_682_944, 151_257_088, 2 ** 32 - 1):
            assert qp.qp_packed_bytes(n, bits) == 4 * ((n * bits + 31) // 32) == orc.packed_bytes(n, bits)
    for bad in (0, 1, 5, 7, 9, 12, 32):
        assert qp.qp_packed_bytes(100, bad) == 0


def test_workspace_bytes(qp):
    cfg = qp.qp_default_search_cfg()
    assert (cfg.t_steps, cfg.cands_per_round, cfg.nbins, cfg.dist, cfg.flags, cfg.coarse_stride) == (100, 13, 2048, qp.QP_LAPLACE, 0, 0)
    a = qp.qp_workspace_bytes(9_682_944)
    assert a == qp.qp_workspace_bytes(9_682_944, cfg) and a > qp.qp_ws_offset(qp.QP_WS_SCORES)
    cfg.t_steps = 1000
    assert qp.qp_workspace_bytes(9_682_944, cfg) > a
    assert qp.qp_workspace_bytes(0) == 0 and qp.qp_workspace_bytes(2 ** 32) == 0
    for t, cpr in ((0, 32), (1024, 32), (100, 0), (100, 33)):
        cfg = qp.qp_default_search_cfg()
        cfg.t_steps, cfg.cands_per_round = t, cpr
        assert qp.qp_workspace_bytes(1000, cfg) == 0


def test_aciq_constants_against_scipy_and_oracle(qp):
    for bits in BITS:
        F = qp.qp_aciq_constant(bits, qp.QP_LAPLACE)
        assert F == pytest.approx(scipy.special.lambertw(3 * 4.0 ** bits).real, rel=1e-14)
        assert F == pytest.approx(orc.laplace_F(bits), rel=1e-14)
        assert qp.qp_aciq_constant(bits, qp.QP_GAUSS) == pytest.approx(orc.gauss_G(bits), rel=1e-12)
    assert math.isnan(qp.qp_aciq_constant(5, 0)) and math.isnan(qp.qp_aciq_constant(4, 7))


def test_aciq_alpha_host(qp):
    st = qp.qp_stats_t()
    st.mad, st.var = 0.37, 0.49
    for bits in BITS:
        assert qp.qp_aciq_alpha(st, bits) == pytest.approx(orc.laplace_F(bits) * 0.37, rel=1e-14)
        assert qp.qp_aciq_alpha(st, bits, qp.QP_GAUSS) == pytest.approx(orc.gauss_G(bits) * 0.7, rel=1e-12)
    with pytest.raises(qp.QuantPipeError):
        qp.qp_aciq_alpha(st, 5)
    with pytest.raises(qp.QuantPipeError):
        qp.qp_aciq_alpha(st, 4, 3)


def test_make_qparams_is_bit_identical_to_the_oracle(qp):
    rng = np.random.default_rng(0)
    for _ in range(3000):
        center = rng.normal(0, 1) * 10.0 ** rng.integers(-6, 6)
        alpha = abs(rng.normal(0, 1)) * 10.0 ** rng.integers(-8, 8)
        bits = int(rng.choice(BITS))
        a = qp.qp_make_qparams(center, alpha, bits, 77)
        b = orc.make_qparams(center, alpha, bits, 77)
        assert (a.lo, a.hi, a.scale, a.inv_scale, a.bits, a.n) == (b.lo, b.hi, b.scale, b.inv_scale, bits, 77)
        assert a.reserved == 0
    z = qp.qp_make_qparams(3.0, 0.0, 4, 1)
    assert (z.lo, z.hi, z.scale, z.inv_scale) == (3.0, 3.0, 0.0, 0.0)
    with pytest.raises(qp.QuantPipeError):
        qp.qp_make_qparams(0.0, 1.0, 7, 1)


def test_argument_errors_are_reported_before_any_gpu_work(qp):
    L = qp.lib()
    fake = C.c_void_p(0x10000)          # aligned, never dereferenced on these paths
    odd = C.c_void_p(0x10004)           # misaligned
    q = qp.qp_make_qparams(0.0, 1.0, 4, 1000)
    st = qp.qp_stats_t()
    big = 1 << 30
    # null pointers / n == 0 / bad dtype / bad nbins / misalignment
    assert L.qp_stats(None, 1000, 0, 2048, fake, big, None, C.byref(st)) == qp.QP_EINVAL
    assert L.qp_stats(fake, 0, 0, 2048, fake, big, None, C.byref(st)) == qp.QP_EINVAL
    assert L.qp_stats(fake, 1000, 2, 2048, fake, big, None, C.byref(st)) == qp.QP_EINVAL
    assert L.qp_stats(fake, 1000, 0, 8, fake, big, None, C.byref(st)) == qp.QP_EINVAL
    assert L.qp_stats(fake, 1000, 0, 5000, fake, big, None, C.byref(st)) == qp.QP_EINVAL
    assert L.qp_stats(odd, 1000, 0, 2048, fake, big, None, C.byref(st)) == qp.QP_EINVAL
    assert L.qp_stats(fake, 1000, 0, 2048, None, big, None, C.byref(st)) == qp.QP_EINVAL
    assert L.qp_stats(fake, 1000, 0, 2048, fake, big, None, None) == qp.QP_EINVAL
    assert L.qp_stats(fake, 2 ** 32, 0, 2048, fake, big, None, C.byref(st)) == qp.QP_EINVAL
    assert L.qp_stats(fake, 1000, 0, 2048, fake, 100, None, C.byref(st)) == qp.QP_ENOSPC
    # search
    res, qo = qp.qp_search_result_t(), qp.qp_qparams_t()
    assert L.qp_dsaciq_search(fake, 1000, 0, None, 4, None, fake, big, None, C.byref(res), C.byref(qo)) == qp.QP_EINVAL
    assert L.qp_dsaciq_search(fake, 1000, 0, C.byref(st), 5, None, fake, big, None, C.byref(res), C.byref(qo)) == qp.QP_EINVAL
    assert L.qp_dsaciq_search(fake, 1000, 0, C.byref(st), 4, None, fake, 1000, None, C.byref(res), C.byref(qo)) == qp.QP_ENOSPC
    for field, value in (("dist", 3), ("flags", 8), ("coarse_stride", 65), ("cands_per_round", 33), ("t_steps", 0)):
        cfg = qp.qp_default_search_cfg()
        setattr(cfg, field, value)
        assert L.qp_dsaciq_search(fake, 1000, 0, C.byref(st), 4, C.byref(cfg), fake, big, None, C.byref(res), C.byref(qo)) == qp.QP_EINVAL, field
    for field, value in (("dist", qp.QP_GAUSS), ("dist", qp.QP_DIST_AUTO), ("flags", qp.QP_SEARCH_CLIP_TO_DATA)):    # the histogram fit is the paper's form only
        cfg = qp.qp_default_search_cfg()
        setattr(cfg, field, value)
        assert L.qp_dsaciq_hist_search_async(4, C.byref(cfg), fake, big, None) == qp.QP_EINVAL, field
    cfg = qp.qp_default_search_cfg()
    cfg.t_steps = 5000
    assert L.qp_dsaciq_search_async(fake, 1000, 0, 4, C.byref(cfg), fake, big, None) == qp.QP_EINVAL
    # model fit: the choice needs the histogram, so the host-only alpha does not take QP_DIST_AUTO
    mf = qp.qp_model_fit_t()
    assert L.qp_model_fit(None, big, None, C.byref(mf)) == qp.QP_EINVAL
    assert L.qp_model_fit(fake, big, None, None) == qp.QP_EINVAL
    assert L.qp_model_fit(odd, big, None, C.byref(mf)) == qp.QP_EINVAL
    assert L.qp_model_fit_async(fake, 64, None) == qp.QP_ENOSPC
    alpha = C.c_double()
    assert L.qp_aciq_alpha(C.byref(st), 4, qp.QP_DIST_AUTO, C.byref(alpha)) == qp.QP_EINVAL
    assert math.isnan(L.qp_aciq_constant(4, qp.QP_DIST_AUTO))
    # histogram-fit search
    assert L.qp_dsaciq_hist_search_async(5, None, fake, big, None) == qp.QP_EINVAL
    assert L.qp_dsaciq_hist_search_async(4, None, None, big, None) == qp.QP_EINVAL
    assert L.qp_dsaciq_hist_search_async(4, None, odd, big, None) == qp.QP_EINVAL
    assert L.qp_dsaciq_hist_search_async(4, None, fake, 1000, None) == qp.QP_ENOSPC
    assert L.qp_dsaciq_hist_search(4, C.byref(cfg), fake, big, None, C.byref(res), C.byref(qo)) == qp.QP_EINVAL   # t_steps 5000
    # pack
    assert L.qp_quant_pack(fake, 1000, 0, None, fake, big, None) == qp.QP_EINVAL
    assert L.qp_quant_pack(fake, 999, 0, C.byref(q), fake, big, None) == qp.QP_EINVAL        # n mismatch
    assert L.qp_quant_pack(fake, 1000, 0, C.byref(q), fake, 499, None) == qp.QP_ENOSPC
    assert L.qp_quant_pack(fake, 1000, 0, C.byref(q), odd, big, None) == qp.QP_EINVAL
    assert L.qp_quant_pack(None, 1000, 0, C.byref(q), fake, big, None) == qp.QP_EINVAL
    bad = qp.qp_make_qparams(0.0, 1.0, 4, 1000)
    bad.bits = 5
    assert L.qp_quant_pack(fake, 1000, 0, C.byref(bad), fake, big, None) == qp.QP_EINVAL
    assert L.qp_quant_pack_dev(fake, 1000, 0, 4, None, fake, big, None) == qp.QP_EINVAL
    # unpack
    assert L.qp_unpack_dequant(fake, big, None, fake, 1000, None) == qp.QP_EINVAL
    assert L.qp_unpack_dequant(fake, big, C.byref(q), fake, 1001, None) == qp.QP_EINVAL
    assert L.qp_unpack_dequant(fake, 499, C.byref(q), fake, 1000, None) == qp.QP_ENOSPC
    assert L.qp_unpack_dequant(fake, big, C.byref(bad), fake, 1000, None) == qp.QP_EINVAL
    assert L.qp_unpack_dequant(fake, big, C.byref(q), None, 1000, None) == qp.QP_EINVAL
    assert L.qp_unpack_dequant_dev(fake, big, 4, None, fake, 1000, None) == qp.QP_EINVAL
    # whole sender side
    assert L.qp_compress_async(fake, 1000, 0, 4, None, fake, big, fake, 499, None, None) == qp.QP_ENOSPC
    assert L.qp_compress_async(fake, 1000, 0, 9, None, fake, big, fake, big, None, None) == qp.QP_EINVAL
    assert L.qp_compress_async(fake, 1000, 0, 4, None, fake, 64, fake, big, None, None) == qp.QP_ENOSPC


def test_strerror(qp):
    msgs = {qp.qp_strerror(s) for s in (0, -1, -2, -3, -4, -99)}
    assert len(msgs) == 6 and qp.qp_strerror(0) == "ok"


def test_product_package_does_not_reach_the_oracle():
    pkg = os.path.join(ROOT, "paper_2211_04515_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "qp_oracle" not in text and "import oracle" not in text and "from oracle" not in text, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            assert "paper_2211_04515_amd" not in open(os.path.join(ROOT, "oracle", f)).read(), f


def test_next_bits_matches_oracle_and_the_papers_example(qp):
    n = 64 * 197 * 768
    for bw, q_expected in ((400e6, 16), (50e6, 2), (200e6, 8), (float("inf"), 32)):
        for q_cur in (32, 16, 8, 6, 4, 3, 2):
            assert qp.qp_next_bits(n * q_cur, q_cur, 64, 100.0, bw) == q_expected
    rng = np.random.default_rng(5)
    for _ in range(3000):
        nn = int(rng.integers(10_000, 50_000_000))
        q_cur = int(rng.choice((2, 3, 4, 6, 8, 16, 32)))
        s_img, rate = float(rng.integers(1, 129)), float(rng.uniform(5, 500))
        bw = float(10 ** rng.uniform(5.0, 11.0))
        assert qp.qp_next_bits(nn * q_cur, q_cur, s_img, rate, bw) == orc.next_bits(nn * q_cur, q_cur, s_img, rate, bw)
    for bad in ((0, 8, 64, 100, 1e8), (1e6, 5, 64, 100, 1e8), (1e6, 8, 0, 100, 1e8), (1e6, 8, 64, -1, 1e8),
                (1e6, 8, 64, 100, 0.0), (float("nan"), 8, 64, 100, 1e8), (1e6, 8, 64, 100, float("nan"))):
        with pytest.raises(qp.QuantPipeError):
            qp.qp_next_bits(*bad)


def test_make_qparams_clipped_is_bit_identical_to_the_oracle(qp):
    rng = np.random.default_rng(9)
    for bits in BITS:
        for _ in range(100):
            center, alpha = float(rng.normal()), float(abs(rng.normal()) * 3)
            lo, hi = sorted((float(rng.normal() * 2), float(rng.normal() * 2)))
            if rng.random() < 0.3:
                lo, hi = min(lo, center - 10), max(hi, center + 10)      # data range wider than the clipping range
            a = qp.qp_make_qparams_clipped(center, alpha, lo, hi, bits, 31)
            b = orc.make_qparams_clipped(center, alpha, lo, hi, bits, 31)
            assert (a.bits, a.n, a.lo, a.hi, a.scale, a.inv_scale) == (b.bits, b.n, b.lo, b.hi, b.scale, b.inv_scale)
    z = qp.qp_make_qparams_clipped(2.0, 1.0, 2.0, 2.0, 4, 3)
    assert (z.lo, z.hi, z.scale, z.inv_scale) == (2.0, 2.0, 0.0, 0.0)
    with pytest.raises(qp.QuantPipeError):
        qp.qp_make_qparams_clipped(0.0, 1.0, -1.0, 1.0, 5, 1)


def test_coarse_to_fine_is_refused_where_it_is_not_offered(qp):
    """bf16 tensors of 2^20 elements or more (searched through their value table): QP_EINVAL before anything is
    launched (no GPU needed)."""
    L = qp.lib()
    fake, big = C.c_void_p(0x1000), 1 << 40
    st, res, qo = qp.qp_stats_t(), qp.qp_search_result_t(), qp.qp_qparams_t()
    cfg = qp.qp_default_search_cfg()
    cfg.flags, cfg.coarse_stride = qp.QP_SEARCH_COARSE_TO_FINE, 10
    for n in (1 << 20, 200_000_000):
        assert L.qp_dsaciq_search(fake, n, qp.QP_BF16, C.byref(st), 4, C.byref(cfg), fake, big, None, C.byref(res), C.byref(qo)) == qp.QP_EINVAL
        assert L.qp_dsaciq_search_async(fake, n, qp.QP_BF16, 4, C.byref(cfg), fake, big, None) == qp.QP_EINVAL
        assert L.qp_compress_async(fake, n, qp.QP_BF16, 4, C.byref(cfg), fake, big, fake, big, None, None) == qp.QP_EINVAL


def test_controller_is_the_oracles_controller(qp):
    """qp_controller_* against the oracle on random traces (same decision after every microbatch) and on the paper's
    five-phase run (Sec. 4.2)."""
    assert C.sizeof(qp.qp_controller_t) == 48
    rng = np.random.default_rng(21)
    for trial in range(40):
        window = int(rng.integers(1, 30))
        s_img, rate = float(rng.integers(1, 65)), float(rng.uniform(10, 300))
        q0 = int(rng.choice([32, 16, 8, 6, 4, 3, 2]))
        a, b = qp.qp_controller_init(window, s_img, rate, q0), orc.controller(window, s_img, rate, q0)
        n = int(rng.integers(100_000, 20_000_000))
        q = q0
        for m in range(window * 5 + 3):
            bits = float(n * q)
            secs = bits / float(10 ** rng.uniform(6.5, 9.5))
            qa, qb = qp.qp_controller_update(a, bits, secs), orc.controller_update(b, bits, secs)
            assert qa == qb and (a.count, a.decisions, a.q_cur) == (b.count, b.decisions, b.q_cur)
            q = qa
    n = 64 * 197 * 768
    c = qp.qp_controller_init(50, 64, 100.0)
    used, q = [], 32
    for bw in (np.inf, 400e6, 50e6, 200e6, np.inf):
        for _ in range(200):
            used.append(q)
            q = qp.qp_controller_update(c, n * q, n * q / bw if np.isfinite(bw) else 1e-6)
    assert [used[200 * p + 199] for p in range(5)] == [32, 16, 2, 8, 32]
    L = qp.lib()
    out = C.c_uint32()
    assert L.qp_controller_init(None, 50, 64.0, 100.0, 32) == qp.QP_EINVAL
    for args in ((0, 64.0, 100.0, 32), (50, 0.0, 100.0, 32), (50, 64.0, -1.0, 32), (50, 64.0, 100.0, 5), (50, float("nan"), 100.0, 32)):
        assert L.qp_controller_init(C.byref(c), *args) == qp.QP_EINVAL, args
    c = qp.qp_controller_init(2, 64, 100.0)
    for bits, secs in ((0.0, 1.0), (1.0, 0.0), (float("nan"), 1.0), (1.0, float("inf"))):
        assert L.qp_controller_update(C.byref(c), bits, secs, C.byref(out)) == qp.QP_EINVAL
    assert (c.count, c.decisions) == (0, 0)
    assert L.qp_controller_update(C.byref(c), 1.0, 1.0, None) == qp.QP_EINVAL
