"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element,
on the same seeded inputs.  Needs a real MI355X: run with -m gpu."""
import ctypes as C
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

import synth_inputs as si
from oracle import qp_oracle as orc

pytestmark = pytest.mark.gpu


def print(*args, **kwargs):
    """The tests' "[case] ..." lines go to the real stderr, unbuffered: a run that faults or hangs has named its case."""
    import builtins
    import sys
    builtins.print(*args, **{**kwargs, "file": sys.__stderr__, "flush": True})

torch = pytest.importorskip("torch")
BITS = (2, 3, 4, 6, 8, 16)

# Tolerances (floating point): statistics and alpha 1e-5 relative is the stated bar; what the
# arithmetic gives is far tighter (fp64 sums that differ only in summation order), and the
# tests hold it to 1e-11 so that a real defect cannot hide inside the bar.
REL_STATS = 1e-11
REL_SCORE = 1e-11
# At full size the oracle's own sequential fp64 sums (10^7 to 10^8 terms) carry up to ~1e-10 of
# rounding error, so the oracle comparison is held to 1e-9 there and the GPU is also checked
# against numpy's pairwise fp64 sums (error ~1e-15) at 1e-12.
REL_STATS_FULL = 1e-9
REL_STATS_PAIRWISE = 1e-12
REL_SCORE_FULL = 1e-9          # same reason: the oracle's sequential sum of ~10^7 squares is off by ~1e-11
REL_SCORE_PAIRWISE = 1e-12


def rel_score_sequential(n):
    """Tolerance against the oracle's term-by-term fp64 sum of n non-negative terms: its a-priori rounding
    bound, n * 2^-53 relative (Eq. 1 fixes no order for the sum).  1.1e-9 at the 9.7 M elements of the
    ViT-Base tensor, 1.7e-8 at the 151 M of the large bf16 one, where that sum was measured 1.2e-9 away
    from the pairwise one; the pairwise sums are the tight check at those sizes."""
    return max(REL_SCORE_FULL, n * 2.0 ** -53)


def pairwise_sq_error(x, oq):
    """Sum of squared errors of the oracle's own quantize/dequantize, added with numpy's pairwise fp64 sum."""
    e = (x - orc.dequantize(orc.quantize(x, oq), oq)).astype(np.float64)
    e *= e
    return float(np.sum(e))


ORACLE_THREADS = 16     # host threads the full-size tests spread the oracle's candidates over
TIES = {"count": 0}     # searches whose winner differed from the oracle's by a numerical tie (expected: none)


def check_winner(x, ost, bits, j_gpu, ores, t_steps=100):
    """The GPU's winner against the oracle's (both from the statistics `ost`).  Equal, or a numerical tie:
    the error of the GPU's candidate, by the oracle's own quantizer and numpy's pairwise fp64 sum (good to
    1e-15, which the oracle's term-by-term sum is not at 10^7 terms), within 1e-12 of the oracle winner's.
    Ties are counted and reported."""
    if j_gpu == ores.j_star:
        return True
    e_gpu = pairwise_sq_error(x, orc.search_candidate(ost, bits, t_steps, x.size, j_gpu))
    e_orc = pairwise_sq_error(x, orc.search_candidate(ost, bits, t_steps, x.size, ores.j_star))
    TIES["count"] += 1
    print(f"[tie] bits={bits}: GPU j*={j_gpu} ({e_gpu!r}), oracle j*={ores.j_star} ({e_orc!r}); ties so far {TIES['count']}", flush=True)
    assert abs(e_gpu - e_orc) <= 1e-12 * e_orc, (bits, j_gpu, ores.j_star, e_gpu, e_orc)
    return False


def check_stats_full(st, ost, x):
    for f in ("mean", "mad", "abs_mean", "var"):
        assert abs(getattr(st, f) - getattr(ost, f)) <= REL_STATS_FULL * max(abs(getattr(ost, f)), 1e-3 * ost.abs_mean), f
    assert (st.min, st.max, st.peak_count) == (ost.min, ost.max, ost.peak_count)
    x64 = x.astype(np.float64)
    mu = float(np.sum(x64)) / x.size
    x64 -= st.mean                       # deviations about the GPU's own mean
    np.abs(x64, out=x64)
    mad = float(np.sum(x64)) / x.size
    x64 *= x64
    var = float(np.sum(x64)) / x.size
    scale = max(abs(mu), 1e-3 * ost.abs_mean)
    assert abs(st.mean - mu) <= REL_STATS_PAIRWISE * scale
    assert abs(st.mad - mad) <= REL_STATS_PAIRWISE * mad and abs(st.var - var) <= REL_STATS_PAIRWISE * var


@pytest.fixture(scope="module")
def qp():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2211_04515_amd as m
    m.lib()
    return m


def to_dev(x):
    """numpy float32 array, or uint16 array of bf16 bit patterns -> device tensor."""
    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16).copy()).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()


def as_f32(x):
    return orc.widen_bf16(x) if x.dtype == np.uint16 else x


def oracle_stats_from(st):
    o = orc.Stats()
    for name, _ in orc.Stats._fields_:
        setattr(o, name, getattr(st, name))
    return o


def oracle_q_from(q):
    return orc.qparams_from_floats(q.bits, q.n, q.lo, q.hi, q.scale, q.inv_scale)


def inputs_small():
    cases = [("C1", si.make_config("C1")),
             ("C2_ragged", si.make_config("C2", n=1_234_567)),
             ("C3_ragged", si.make_config("C3", n=987_653)),
             ("C4_scaled", (si.make_config("C4", n=300_001) * np.float32(1.7))),
             ("C5_bf16", si.make_config("C5", n=777_779))]
    cases += si.edge_cases()
    return cases


SMALL = inputs_small()
SMALL_IDS = [c[0] for c in SMALL]


# ----------------------------------------------------------------------------- step 1

@pytest.mark.parametrize("name,x", SMALL, ids=SMALL_IDS)
def test_stats_match_oracle(qp, name, x):
    print(f"[case] stats {name} n={x.size}", flush=True)
    xd = to_dev(x)
    ws = qp.alloc_workspace(x.size)
    st = qp.qp_stats(xd, ws)
    rc, ref, hist_ref = orc.stats(as_f32(x), want_hist=True)
    assert rc == 0
    assert st.n == ref.n == x.size and st.n_nonfinite == 0
    assert st.min == ref.min and st.max == ref.max
    for f in ("mean", "mad", "abs_mean", "var"):
        a, b = getattr(st, f), getattr(ref, f)
        scale = max(abs(b), ref.abs_mean * 1e-3 if f == "mean" else 0.0)
        assert abs(a - b) <= REL_STATS * scale + 0.0, (f, a, b)
    off = qp.qp_ws_offset(qp.QP_WS_HIST)
    hist = ws[off:off + 4 * 2048].cpu().numpy().view(np.uint32)
    assert np.array_equal(hist, hist_ref[:2048])           # integer work: exact
    assert st.peak_count == ref.peak_count and st.nbins == 2048
    assert st.peak_density == pytest.approx(ref.peak_density, rel=1e-14)
    assert st.b_r == pytest.approx(ref.b_r, rel=1e-14)


def test_stats_other_bin_counts(qp):
    x = si.make_config("C2", n=200_003)
    xd = to_dev(x)
    ws = qp.alloc_workspace(x.size)
    for nbins in (16, 100, 4096):
        st = qp.qp_stats(xd, ws, nbins=nbins)
        rc, ref, hist_ref = orc.stats(x, nbins=nbins, want_hist=True)
        off = qp.qp_ws_offset(qp.QP_WS_HIST)
        hist = ws[off:off + 4 * nbins].cpu().numpy().view(np.uint32)
        assert np.array_equal(hist, hist_ref[:nbins])
        assert st.peak_count == ref.peak_count and st.b_r == pytest.approx(ref.b_r, rel=1e-14)


def test_stats_nonfinite_is_an_error(qp):
    x = si.make_config("C1").copy()
    x[5] = np.nan
    x[77777] = -np.inf
    xd = to_dev(x)
    ws = qp.alloc_workspace(x.size)
    with pytest.raises(qp.QuantPipeError) as e:
        qp.qp_stats(xd, ws)
    assert e.value.status == qp.QP_ENONFINITE
    st = qp.qp_stats(xd, ws, allow_nonfinite=True)
    assert st.n_nonfinite == 2


def test_stats_are_bit_reproducible(qp):
    x = si.make_config("C3", n=2_000_003)
    xd = to_dev(x)
    ws = qp.alloc_workspace(x.size)
    first = bytes(qp.qp_stats(xd, ws))
    for _ in range(10):
        assert bytes(qp.qp_stats(xd, ws)) == first


# ----------------------------------------------------------------------------- step 2

def test_aciq_alpha_matches_oracle(qp):
    x = si.make_config("C1")
    ws = qp.alloc_workspace(x.size)
    st = qp.qp_stats(to_dev(x), ws)
    ost = oracle_stats_from(st)
    for bits in BITS:
        assert qp.qp_aciq_alpha(st, bits) == pytest.approx(orc.aciq_alpha(ost, bits), rel=1e-14)
        assert qp.qp_aciq_alpha(st, bits, qp.QP_GAUSS) == pytest.approx(orc.aciq_alpha(ost, bits, orc.GAUSS), rel=1e-12)


SEARCH_CASES = [("C1", None, (2, 4, 8)), ("C2", 300_007, BITS), ("C3", 250_001, (2, 4, 8)),
                ("C4", 200_000, (2, 6, 16)), ("C5", 300_011, (2, 3, 4, 8)),
                # large bf16 tensors are searched through their value table
                ("C5", 1_200_003, (2, 8))]


@pytest.mark.parametrize("name,n,bitset", SEARCH_CASES, ids=[f"{c[0]}_{c[1]}" for c in SEARCH_CASES])
def test_search_matches_oracle(qp, name, n, bitset):
    x = si.make_config(name, n=n)
    xf = as_f32(x)
    xd = to_dev(x)
    ws = qp.alloc_workspace(x.size)
    st = qp.qp_stats(xd, ws)
    rc, ost_own = orc.stats(xf)
    cfg = qp.qp_default_search_cfg()
    if name == "C3":
        cfg.cands_per_round = 32     # this configuration names 32 candidates per search round
    for bits in bitset:
        print(f"[case] search {name} n={x.size} bits={bits}", flush=True)
        res, q = qp.qp_dsaciq_search(xd, st, bits, ws, cfg=cfg)
        off = qp.qp_ws_offset(qp.QP_WS_SCORES)
        scores = ws[off:off + 8 * 101].cpu().numpy().view(np.float64)
        # (i) oracle given the GPU's statistics: same grid, so scores differ only by summation order
        ores, oq, oscores = orc.dsaciq_search(xf, oracle_stats_from(st), bits, 100)
        # the oracle adds its 10^6 terms one after the other, which alone costs it about 1e-11
        # (measured against the exactly rounded sum); the pairwise sum below is the tight check there
        tol = REL_SCORE if x.size < (1 << 19) else REL_SCORE_FULL
        assert np.allclose(scores, oscores, rtol=tol, atol=0.0)
        if x.size >= (1 << 19):
            F = orc.laplace_F(bits)
            for j in (0, 37, 100):
                oqj = orc.make_qparams(st.mean, F * (st.mad + j * ((st.b_r - st.mad) / 100)), bits, x.size)
                assert scores[j] == pytest.approx(pairwise_sq_error(xf, oqj), rel=REL_SCORE_PAIRWISE)
        if check_winner(xf, oracle_stats_from(st), bits, res.j_star, ores):   # only a numerical tie may differ
            assert res.alpha_star == pytest.approx(ores.alpha_star, rel=1e-14)
            assert (q.lo, q.hi, q.scale, q.inv_scale) == (oq.lo, oq.hi, oq.scale, oq.inv_scale)
        assert res.mse_star == pytest.approx(ores.mse_star, rel=tol)
        assert res.mse_aciq == pytest.approx(ores.mse_aciq, rel=tol)
        assert res.mse_star <= res.mse_aciq and res.t_steps == 100
        assert (q.bits, q.n) == (bits, x.size)
        # (ii) oracle end to end from its own statistics: the stated bar, 1e-5 relative on alpha.  Equal
        # winner: the alphas agree to 1e-5; a different winner must be a numerical tie on the oracle's side
        ores2, _, _ = orc.dsaciq_search(xf, ost_own, bits, 100)
        if check_winner(xf, ost_own, bits, res.j_star, ores2):
            assert res.alpha_star == pytest.approx(ores2.alpha_star, rel=1e-5)
        print(f"[ties] {TIES['count']} so far", flush=True)
        # the candidate table itself
        offc = qp.qp_ws_offset(qp.QP_WS_CANDS)
        cands = ws[offc:offc + 16 * 101].cpu().numpy().view(np.float32).reshape(101, 4)
        F = orc.laplace_F(bits)
        for j in (0, 1, 50, 100):
            b = st.mad + j * ((st.b_r - st.mad) / 100)
            oqj = orc.make_qparams(st.mean, F * b, bits, x.size)
            assert tuple(cands[j]) == (oqj.lo, oqj.hi, oqj.scale, oqj.inv_scale)


def test_search_result_does_not_depend_on_candidates_per_round(qp):
    x = si.make_config("C3", n=150_001)
    xd = to_dev(x)
    ws = qp.alloc_workspace(x.size)
    st = qp.qp_stats(xd, ws)
    off = qp.qp_ws_offset(qp.QP_WS_SCORES)
    ref = None
    for cpr in (32, 1, 7, 16, 25):
        cfg = qp.qp_default_search_cfg()
        cfg.cands_per_round = cpr
        res, q = qp.qp_dsaciq_search(xd, st, 4, ws, cfg=cfg)
        scores = ws[off:off + 8 * 101].cpu().numpy().view(np.float64).copy()
        if ref is None:
            ref = (scores, res.j_star, bytes(q))
        else:
            # the block grid depends on the number of rounds, so only the order of the fp64 sums may differ
            assert np.allclose(scores, ref[0], rtol=1e-13, atol=0.0) and res.j_star == ref[1] and bytes(q) == ref[2]


def test_streaming_search_round_sizes(qp):
    """A tensor large enough for the streaming kernel: every round size it is built for (16, 13, 8, 4, 2, 1
    candidates per round, chosen from cands_per_round) gives the same scores up to the order of the sums."""
    x = si.make_config("C2", n=2_300_011)
    xd = to_dev(x)
    off = qp.qp_ws_offset(qp.QP_WS_SCORES)
    for t, cprs in ((100, (13, 32, 8, 5, 3, 1)), (111, (13, 16))):
        ref = None
        for cpr in cprs:
            print(f"[case] round sizes t={t} cands_per_round={cpr}", flush=True)
            cfg = qp.qp_default_search_cfg()
            cfg.t_steps, cfg.cands_per_round = t, cpr
            ws = qp.alloc_workspace(x.size, cfg)
            st = qp.qp_stats(xd, ws)
            res, q = qp.qp_dsaciq_search(xd, st, 3, ws, cfg=cfg)
            scores = ws[off:off + 8 * (t + 1)].cpu().numpy().view(np.float64).copy()
            if ref is None:
                ref = (scores, res.j_star, bytes(q))
                oqj = orc.make_qparams(st.mean, orc.laplace_F(3) * (st.mad + t * ((st.b_r - st.mad) / t)), 3, x.size)
                assert scores[t] == pytest.approx(pairwise_sq_error(x, oqj), rel=REL_SCORE_PAIRWISE)
            else:
                assert np.allclose(scores, ref[0], rtol=1e-13, atol=0.0) and res.j_star == ref[1] and bytes(q) == ref[2]


def test_search_other_step_counts(qp):
    x = si.make_config("C3", n=60_001)
    xd = to_dev(x)
    st = None
    for t in (1, 10, 333, 1023):
        cfg = qp.qp_default_search_cfg()
        cfg.t_steps = t
        ws = qp.alloc_workspace(x.size, cfg)
        st = qp.qp_stats(xd, ws)
        res, q = qp.qp_dsaciq_search(xd, st, 2, ws, cfg=cfg)
        ores, oq, oscores = orc.dsaciq_search(x, oracle_stats_from(st), 2, t)
        off = qp.qp_ws_offset(qp.QP_WS_SCORES)
        scores = ws[off:off + 8 * (t + 1)].cpu().numpy().view(np.float64)
        assert np.allclose(scores, oscores, rtol=REL_SCORE, atol=0.0)
        assert res.j_star == ores.j_star and res.t_steps == t


def test_search_short_sweep_on_a_large_tensor(qp):
    # a sweep that fits one round of candidates (t + 1 <= cands_per_round) is scored by the tile search
    # whatever the tensor's size
    x = si.make_config("C3", n=2_600_011)
    xd = to_dev(x)
    cfg = qp.qp_default_search_cfg()
    cfg.t_steps = 10
    assert cfg.t_steps + 1 <= cfg.cands_per_round
    ws = qp.alloc_workspace(x.size, cfg)
    st = qp.qp_stats(xd, ws)
    for bits in (2, 4):
        print(f"[case] short sweep n={x.size} t={cfg.t_steps} bits={bits}", flush=True)
        res, q = qp.qp_dsaciq_search(xd, st, bits, ws, cfg=cfg)
        ores, oq, oscores = orc.dsaciq_search(x, oracle_stats_from(st), bits, cfg.t_steps)
        off = qp.qp_ws_offset(qp.QP_WS_SCORES)
        scores = ws[off:off + 8 * (cfg.t_steps + 1)].cpu().numpy().view(np.float64)
        assert np.allclose(scores, oscores, rtol=REL_SCORE_FULL, atol=0.0)
        assert res.j_star == ores.j_star and res.t_steps == cfg.t_steps
        assert (q.lo, q.hi, q.scale, q.inv_scale) == (oq.lo, oq.hi, oq.scale, oq.inv_scale)


@pytest.mark.parametrize("name", ["constant", "zeros", "two_point", "laplace_n1", "laplace_n5", "subnormal_values",
                                  "tiny_values", "large_values", "huge_outlier"])
def test_search_degenerate_inputs(qp, name):
    x = dict(si.edge_cases())[name]
    xd = to_dev(x)
    ws = qp.alloc_workspace(x.size)
    st = qp.qp_stats(xd, ws)
    res, q = qp.qp_dsaciq_search(xd, st, 4, ws)
    ores, oq, oscores = orc.dsaciq_search(x, oracle_stats_from(st), 4, 100)
    off = qp.qp_ws_offset(qp.QP_WS_SCORES)
    scores = ws[off:off + 8 * 101].cpu().numpy().view(np.float64)
    assert np.allclose(scores, oscores, rtol=REL_SCORE, atol=0.0, equal_nan=True)
    assert res.j_star == ores.j_star
    assert (q.lo, q.hi, q.scale, q.inv_scale) == (oq.lo, oq.hi, oq.scale, oq.inv_scale)


def test_search_is_bit_reproducible(qp):
    x = si.make_config("C2", n=1_000_003)
    xd = to_dev(x)
    ws = qp.alloc_workspace(x.size)
    st = qp.qp_stats(xd, ws)
    off = qp.qp_ws_offset(qp.QP_WS_SCORES)
    first = None
    for _ in range(5):
        res, q = qp.qp_dsaciq_search(xd, st, 3, ws)
        cur = (ws[off:off + 8 * 101].cpu().numpy().tobytes(), bytes(res), bytes(q))
        first = first or cur
        assert cur == first


# ----------------------------------------------------------------------------- steps 3 and 4

def gpu_alpha_qparams(qp, x, xd, bits, ws):
    st = qp.qp_stats(xd, ws)
    alpha = qp.qp_aciq_alpha(st, bits)
    return qp.qp_make_qparams(st.mean, alpha, bits, x.size), st, alpha


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("name,x", SMALL, ids=SMALL_IDS)
def test_pack_and_unpack_match_oracle(qp, name, x, bits):
    print(f"[case] pack/unpack {name} n={x.size} bits={bits}", flush=True)
    xf = as_f32(x)
    xd = to_dev(x)
    ws = qp.alloc_workspace(x.size)
    q, st, alpha = gpu_alpha_qparams(qp, x, xd, bits, ws)
    # the oracle is given the GPU's alpha and builds its own grid from it: must be the same floats
    oq = orc.make_qparams(st.mean, alpha, bits, x.size)
    assert (q.lo, q.hi, q.scale, q.inv_scale) == (oq.lo, oq.hi, oq.scale, oq.inv_scale)
    packed = qp.alloc_packed(x.size, bits)
    packed.fill_(0xAB)                                   # tail bits must be overwritten with zeros
    qp.qp_quant_pack(xd, q, packed)
    codes_ref = orc.quantize(xf, oq)
    ref = orc.pack(codes_ref, bits)
    got = packed.cpu().numpy()
    assert got.size == ref.size == 4 * ((x.size * bits + 31) // 32)
    assert np.array_equal(got, ref)                      # bit-exact
    y = torch.full((x.size,), float("nan"), dtype=torch.float32, device="cuda")
    qp.qp_unpack_dequant(packed, q, y)
    yref = orc.dequantize(codes_ref, oq)
    assert np.array_equal(y.cpu().numpy().view(np.uint32), yref.view(np.uint32))   # 0 ulp (bar: 1 ulp)


@pytest.mark.parametrize("bits", BITS)
def test_unpack_of_oracle_stream_with_random_codes(qp, bits):
    rng = np.random.default_rng(bits)
    for n in (1, 2, 3, 4, 5, 7, 31, 33, 1021, 8191, 8192, 8193, 32768, 32771, 100_003):
        codes = rng.integers(0, 2 ** bits, size=n, dtype=np.uint32)
        stream = orc.pack(codes, bits)
        oq = orc.make_qparams(-0.3, 2.2, bits, n)
        q = qp.qp_make_qparams(-0.3, 2.2, bits, n)
        pd = torch.from_numpy(stream).cuda()
        y = torch.empty(n, dtype=torch.float32, device="cuda")
        qp.qp_unpack_dequant(pd, q, y)
        assert np.array_equal(y.cpu().numpy(), orc.dequantize(codes, oq)), (bits, n)


@pytest.mark.parametrize("bits", BITS)
def test_pack_special_values_and_naive_range(qp, bits):
    x = si.make_config("C1").copy()
    x[:6] = [np.nan, np.inf, -np.inf, 0.0, -0.0, 1e-40]
    xd = to_dev(x)
    ws = qp.alloc_workspace(x.size)
    x_fin = x.copy()
    x_fin[:3] = 0
    rc, ost = orc.stats(x_fin)
    for center, alpha in ((ost.mean, orc.aciq_alpha(ost, bits)), ((ost.min + ost.max) / 2, (ost.max - ost.min) / 2)):
        q = qp.qp_make_qparams(center, alpha, bits, x.size)
        oq = orc.make_qparams(center, alpha, bits, x.size)
        packed = qp.alloc_packed(x.size, bits)
        qp.qp_quant_pack(xd, q, packed)
        assert np.array_equal(packed.cpu().numpy(), orc.pack(orc.quantize(x, oq), bits))


@pytest.mark.parametrize("bits", (2, 3, 16))
def test_pack_degenerate_grid(qp, bits):
    x = si.make_config("C1")
    xd = to_dev(x)
    q = qp.qp_make_qparams(0.5, 0.0, bits, x.size)
    packed = qp.alloc_packed(x.size, bits)
    packed.fill_(0xFF)
    qp.qp_quant_pack(xd, q, packed)
    assert int(packed.max()) == 0
    y = torch.empty(x.size, dtype=torch.float32, device="cuda")
    qp.qp_unpack_dequant(packed, q, y)
    assert bool((y == 0.5).all())


@pytest.mark.timeout(600)
@pytest.mark.parametrize("kind", ["fp32", "bf16"])
@pytest.mark.parametrize("n", [(1 << 24) - 3, (1 << 24) + 4099])
def test_pack_and_unpack_forms_around_two_to_the_24(qp, kind, n):
    """From 2^24 elements on the launchers take other forms of the same kernels (3- and 6-bit quantize+pack restaged
    through LDS, 512-lane unpack): every bitwidth on both sides of the threshold, whole stream against the oracle."""
    x = si.make_config("C5" if kind == "bf16" else "C2", n=n)
    xf = as_f32(x)
    xd = to_dev(x)
    y = torch.empty(n, dtype=torch.float32, device="cuda")
    for bits in BITS:
        oq = orc.make_qparams(0.03, 1.9, bits, n)
        q = qp.qp_make_qparams(0.03, 1.9, bits, n)
        assert (q.lo, q.hi, q.scale, q.inv_scale) == (oq.lo, oq.hi, oq.scale, oq.inv_scale)
        packed = qp.alloc_packed(n, bits)
        packed.fill_(0xA5)
        qp.qp_quant_pack(xd, q, packed)
        codes = orc.quantize(xf, oq)
        assert np.array_equal(packed.cpu().numpy(), orc.pack(codes, bits)), bits
        y.fill_(float("nan"))
        qp.qp_unpack_dequant(packed, q, y)
        assert np.array_equal(y.cpu().numpy(), orc.dequantize(codes, oq)), bits
        del packed


def test_device_resident_path_matches_host_path(qp):
    x = si.make_config("C3", n=500_009)
    xd = to_dev(x)
    ws = qp.alloc_workspace(x.size)
    for bits in (2, 6):
        st = qp.qp_stats(xd, ws)
        res, q = qp.qp_dsaciq_search(xd, st, bits, ws)
        p_host = qp.alloc_packed(x.size, bits)
        qp.qp_quant_pack(xd, q, p_host)
        y_host = torch.empty(x.size, dtype=torch.float32, device="cuda")
        qp.qp_unpack_dequant(p_host, q, y_host)
        ws2 = qp.alloc_workspace(x.size)
        ws2.fill_(0x5A)                                  # the workspace needs no initialisation
        p_dev = qp.alloc_packed(x.size, bits)
        qrec = torch.zeros(32, dtype=torch.uint8, device="cuda")
        qp.qp_compress_async(xd, bits, ws2, p_dev, qparams_out_dev_ptr=qrec.data_ptr())
        y_dev = torch.empty(x.size, dtype=torch.float32, device="cuda")
        qp.qp_unpack_dequant_dev(p_dev, bits, qrec.data_ptr(), y_dev)
        torch.cuda.synchronize()
        assert torch.equal(p_host, p_dev) and torch.equal(y_host, y_dev)
        assert bytes(qrec.cpu().numpy().tobytes()) == bytes(q)
        assert bytes(qp.read_ws(ws2, qp.QP_WS_STATS, qp.qp_stats_t)) == bytes(st)
        assert bytes(qp.read_ws(ws2, qp.QP_WS_RESULT, qp.qp_search_result_t)) == bytes(res)


def test_runs_on_a_side_stream(qp):
    x = si.make_config("C2", n=400_001)
    xd = to_dev(x)
    ws = qp.alloc_workspace(x.size)
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        st = qp.qp_stats(xd, ws)
        res, q = qp.qp_dsaciq_search(xd, st, 4, ws)
        packed = qp.alloc_packed(x.size, 4)
        qp.qp_quant_pack(xd, q, packed)
    s.synchronize()
    oq = oracle_q_from(q)
    assert np.array_equal(packed.cpu().numpy(), orc.pack(orc.quantize(x, oq), 4))


# ----------------------------------------------------------------------------- full sizes

@pytest.mark.timeout(900)
@pytest.mark.parametrize("name", ["C2", "C3", "C4"])
def test_full_size_fp32_configs(qp, name):
    x = si.make_config(name)
    if name == "C4":
        x = x * np.float32(si.c4_stream(1)[0][1])
    xd = to_dev(x)
    ws = qp.alloc_workspace(x.size)
    st = qp.qp_stats(xd, ws)
    rc, ost, hist_ref = orc.stats(x, want_hist=True)
    check_stats_full(st, ost, x)
    off = qp.qp_ws_offset(qp.QP_WS_HIST)
    assert np.array_equal(ws[off:off + 8192].cpu().numpy().view(np.uint32), hist_ref[:2048])
    offs = qp.qp_ws_offset(qp.QP_WS_SCORES)
    cfg = qp.qp_default_search_cfg()
    if name == "C3":
        cfg.cands_per_round = 32     # this configuration names 32 candidates per search round
    for bits in si.CONFIG_BITS[name]:
        print(f"[case] full {name} bits={bits}", flush=True)
        res, q = qp.qp_dsaciq_search(xd, st, bits, ws, cfg=cfg)
        scores = ws[offs:offs + 8 * 101].cpu().numpy().view(np.float64).copy()
        F = orc.laplace_F(bits)
        # the oracle's whole search at every bitwidth (its 101 candidates spread over host threads): all
        # scores, the winner, alpha and the winner's grid
        ores, oq_s, oscores = orc.dsaciq_search_threads(x, oracle_stats_from(st), bits, 100, ORACLE_THREADS)
        assert np.allclose(scores, oscores, rtol=REL_SCORE_FULL, atol=0.0)
        if check_winner(x, oracle_stats_from(st), bits, res.j_star, ores):
            assert res.alpha_star == pytest.approx(ores.alpha_star, rel=1e-14)
            assert (q.lo, q.hi, q.scale, q.inv_scale) == (oq_s.lo, oq_s.hi, oq_s.scale, oq_s.inv_scale)
        # end to end from the oracle's own statistics: the stated bar, alpha within 1e-5
        ores2, _, _ = orc.dsaciq_search_threads(x, ost, bits, 100, ORACLE_THREADS)
        if check_winner(x, ost, bits, res.j_star, ores2):
            assert res.alpha_star == pytest.approx(ores2.alpha_star, rel=1e-5)
        for j in sorted({0, 100, int(res.j_star)}):
            b = st.mad + j * ((st.b_r - st.mad) / 100)
            oqj = orc.make_qparams(st.mean, F * b, bits, x.size)
            assert scores[j] == pytest.approx(pairwise_sq_error(x, oqj), rel=REL_SCORE_PAIRWISE)
        oq = orc.make_qparams(st.mean, res.alpha_star, bits, x.size)   # oracle given the GPU's alpha
        assert (q.lo, q.hi, q.scale, q.inv_scale) == (oq.lo, oq.hi, oq.scale, oq.inv_scale)
        packed = qp.alloc_packed(x.size, bits)
        qp.qp_quant_pack(xd, q, packed)
        codes = orc.quantize(x, oq)
        assert np.array_equal(packed.cpu().numpy(), orc.pack(codes, bits))
        y = torch.empty(x.size, dtype=torch.float32, device="cuda")
        qp.qp_unpack_dequant(packed, q, y)
        assert np.array_equal(y.cpu().numpy(), orc.dequantize(codes, oq))


@pytest.mark.timeout(1200)
def test_full_size_bf16_config(qp):
    h = si.make_config("C5")
    x = orc.widen_bf16(h)
    xd = to_dev(h)
    ws = qp.alloc_workspace(h.size)
    st = qp.qp_stats(xd, ws)
    rc, ost, hist_ref = orc.stats(x, want_hist=True)
    check_stats_full(st, ost, x)
    off = qp.qp_ws_offset(qp.QP_WS_HIST)
    assert np.array_equal(ws[off:off + 8192].cpu().numpy().view(np.uint32), hist_ref[:2048])
    offs = qp.qp_ws_offset(qp.QP_WS_SCORES)
    for bits in si.CONFIG_BITS["C5"]:
        print(f"[case] full C5 bits={bits}", flush=True)
        res, q = qp.qp_dsaciq_search(xd, st, bits, ws)
        scores = ws[offs:offs + 8 * 101].cpu().numpy().view(np.float64).copy()
        F = orc.laplace_F(bits)
        # the oracle's whole search over the 151 M elements at every bitwidth (candidates spread over host threads)
        ores, oq_s, oscores = orc.dsaciq_search_threads(x, oracle_stats_from(st), bits, 100, ORACLE_THREADS)
        assert np.allclose(scores, oscores, rtol=rel_score_sequential(x.size), atol=0.0)
        if check_winner(x, oracle_stats_from(st), bits, res.j_star, ores):
            assert res.alpha_star == pytest.approx(ores.alpha_star, rel=1e-14)
            assert (q.lo, q.hi, q.scale, q.inv_scale) == (oq_s.lo, oq_s.hi, oq_s.scale, oq_s.inv_scale)
        ores2, _, _ = orc.dsaciq_search_threads(x, ost, bits, 100, ORACLE_THREADS)   # from the oracle's own statistics
        if check_winner(x, ost, bits, res.j_star, ores2):
            assert res.alpha_star == pytest.approx(ores2.alpha_star, rel=1e-5)
        # the tight check at this size: the oracle's quantizer with numpy's pairwise fp64 sum, on candidates
        # spread over the grid (a few at a time: each evaluation holds 2.4 GB of temporaries)
        js = sorted({0, 20, 40, 60, 80, 100, int(res.j_star)})
        with ThreadPoolExecutor(max_workers=4) as ex:
            exact = list(ex.map(lambda j: pairwise_sq_error(x, orc.search_candidate(oracle_stats_from(st), bits, 100, x.size, j)), js))
        for j, e in zip(js, exact):
            assert scores[j] == pytest.approx(e, rel=REL_SCORE_PAIRWISE), j
        print(f"[ties] {TIES['count']} so far", flush=True)
        oq = orc.make_qparams(st.mean, res.alpha_star, bits, x.size)
        packed = qp.alloc_packed(x.size, bits)
        qp.qp_quant_pack(xd, q, packed)
        codes = orc.quantize(x, oq)
        assert np.array_equal(packed.cpu().numpy(), orc.pack(codes, bits))
        y = torch.empty(x.size, dtype=torch.float32, device="cuda")
        qp.qp_unpack_dequant(packed, q, y)
        assert np.array_equal(y.cpu().numpy(), orc.dequantize(codes, oq))
        del packed, y, codes


# ----------------------------------------------------------------------------- the microbatch stream

@pytest.mark.timeout(900)
def test_c4_stream_first_microbatches(qp):
    """Config 4: a stream of microbatches whose bitwidth follows a bandwidth trace; whole sender path
    per microbatch with no host round trip, then the receiver; checked against the oracle."""
    n = si.numel("C4")
    stream = si.c4_stream(40)
    ring = {}
    ws = qp.alloc_workspace(n)
    y = torch.empty(n, dtype=torch.float32, device="cuda")
    qrec = torch.zeros(32, dtype=torch.uint8, device="cuda")
    seen_bits = set()
    checked = 0
    for m, (buf, b_m, bw, bits) in enumerate(stream):
        if bits in seen_bits and checked >= 5:
            continue
        if buf not in ring:
            ring[buf] = si.unit_laplace(n, 100 + buf)
        x = ring[buf] * np.float32(b_m)
        print(f"[case] C4 microbatch {m}: buffer {buf} b={b_m:.3f} bw={bw:.1f} Mbit/s bits={bits}", flush=True)
        xd = to_dev(x)
        packed = qp.alloc_packed(n, bits)
        qp.qp_compress_async(xd, bits, ws, packed, qparams_out_dev_ptr=qrec.data_ptr())
        qp.qp_unpack_dequant_dev(packed, bits, qrec.data_ptr(), y)
        torch.cuda.synchronize()
        q = qp.qp_qparams_t.from_buffer_copy(qrec.cpu().numpy().tobytes())
        res = qp.read_ws(ws, qp.QP_WS_RESULT, qp.qp_search_result_t)
        st = qp.read_ws(ws, qp.QP_WS_STATS, qp.qp_stats_t)
        assert (q.bits, q.n) == (bits, n)
        rc, ost = orc.stats(x)
        assert abs(st.mad - ost.mad) <= REL_STATS_FULL * ost.mad and (st.min, st.max) == (ost.min, ost.max)
        oq = orc.make_qparams(st.mean, res.alpha_star, bits, n)          # the oracle is given the GPU's alpha
        assert (q.lo, q.hi, q.scale, q.inv_scale) == (oq.lo, oq.hi, oq.scale, oq.inv_scale)
        codes = orc.quantize(x, oq)
        assert np.array_equal(packed.cpu().numpy(), orc.pack(codes, bits))
        assert np.array_equal(y.cpu().numpy(), orc.dequantize(codes, oq))
        F = orc.laplace_F(bits)
        b_star = st.mad + res.j_star * ((st.b_r - st.mad) / 100)
        assert res.alpha_star == pytest.approx(F * b_star, rel=1e-14)
        assert res.mse_star == pytest.approx(pairwise_sq_error(x, oq) / n, rel=REL_SCORE_PAIRWISE)
        # the oracle's whole search from the GPU's statistics: every score and the winner
        offs = qp.qp_ws_offset(qp.QP_WS_SCORES)
        scores = ws[offs:offs + 8 * 101].cpu().numpy().view(np.float64)
        ores, _, oscores = orc.dsaciq_search_threads(x, oracle_stats_from(st), bits, 100, ORACLE_THREADS)
        assert np.allclose(scores, oscores, rtol=REL_SCORE_FULL, atol=0.0)
        if check_winner(x, oracle_stats_from(st), bits, res.j_star, ores):
            assert res.alpha_star == pytest.approx(ores.alpha_star, rel=1e-14)
        seen_bits.add(bits)
        checked += 1
    assert checked >= 5 and len(seen_bits) >= 3


@pytest.mark.timeout(900)
def test_timed_step_configuration_on_c2(qp):
    """The step the benchmark times: on the full ViT-Base tensor, for each of its six bitwidths, the sender
    path (statistics, search, pack; parameters stay on the device) and the receiver, back to back on one
    stream with one workspace; the results of every pass are checked against the oracle afterwards."""
    x = si.make_config("C2")
    n = x.size
    xd = to_dev(x)
    ws = qp.alloc_workspace(n)
    bitset = si.CONFIG_BITS["C2"]
    packs = {b: qp.alloc_packed(n, b) for b in bitset}
    ys = {b: torch.empty(n, dtype=torch.float32, device="cuda") for b in bitset}
    recs = {b: torch.zeros(32 + 56 + 8 * 101, dtype=torch.uint8, device="cuda") for b in bitset}
    offr, offs = qp.qp_ws_offset(qp.QP_WS_RESULT), qp.qp_ws_offset(qp.QP_WS_SCORES)
    for b in bitset:   # no synchronisation in between: what a pass leaves is copied aside on the same stream
        qp.qp_compress_async(xd, b, ws, packs[b], qparams_out_dev_ptr=recs[b].data_ptr())
        qp.qp_unpack_dequant_dev(packs[b], b, recs[b].data_ptr(), ys[b])
        recs[b][32:32 + 56].copy_(ws[offr:offr + 56])
        recs[b][88:88 + 808].copy_(ws[offs:offs + 808])
    torch.cuda.synchronize()
    st = qp.read_ws(ws, qp.QP_WS_STATS, qp.qp_stats_t)
    rc, ost = orc.stats(x)
    check_stats_full(st, ost, x)
    for b in bitset:
        print(f"[case] timed step C2 bits={b}", flush=True)
        raw = recs[b].cpu().numpy().tobytes()
        q = qp.qp_qparams_t.from_buffer_copy(raw[:32])
        res = qp.qp_search_result_t.from_buffer_copy(raw[32:88])
        scores = np.frombuffer(raw[88:], dtype=np.float64)
        assert (q.bits, q.n, res.t_steps) == (b, n, 100)
        ores, oq_s, oscores = orc.dsaciq_search_threads(x, oracle_stats_from(st), b, 100, ORACLE_THREADS)
        assert np.allclose(scores, oscores, rtol=REL_SCORE_FULL, atol=0.0)
        if check_winner(x, oracle_stats_from(st), b, res.j_star, ores):
            assert res.alpha_star == pytest.approx(ores.alpha_star, rel=1e-14)
        F = orc.laplace_F(b)
        for j in sorted({0, 100, int(res.j_star)}):
            oqj = orc.make_qparams(st.mean, F * (st.mad + j * ((st.b_r - st.mad) / 100)), b, n)
            assert scores[j] == pytest.approx(pairwise_sq_error(x, oqj), rel=REL_SCORE_PAIRWISE)
        oq = orc.make_qparams(st.mean, res.alpha_star, b, n)   # the oracle is given the GPU's alpha
        assert (q.lo, q.hi, q.scale, q.inv_scale) == (oq.lo, oq.hi, oq.scale, oq.inv_scale)
        codes = orc.quantize(x, oq)
        assert np.array_equal(packs[b].cpu().numpy(), orc.pack(codes, b))
        assert np.array_equal(ys[b].cpu().numpy(), orc.dequantize(codes, oq))


# ----------------------------------------------------------------------------- maximum size

@pytest.mark.timeout(1500)
def test_largest_supported_tensor(qp):
    """n = 2^32 - 1 bf16 elements (8.6 GB in, 17 GB out): 64-bit indexing everywhere, ragged tail."""
    n = 2 ** 32 - 1
    rng = np.random.default_rng(99)
    block = si.f32_to_bf16_bits(rng.laplace(0.0, 0.6, size=1 << 22).astype(np.float32))
    h = np.tile(block, (n + block.size - 1) // block.size)[:n]
    h[12345] = si.f32_to_bf16_bits(np.array([40.0], np.float32))[0]     # the maximum
    h[n - 2] = si.f32_to_bf16_bits(np.array([-37.0], np.float32))[0]    # the minimum, in the tail
    print("[case] largest tensor: upload", flush=True)
    xd = torch.from_numpy(h.view(np.int16)).cuda().view(torch.bfloat16)
    ws = qp.alloc_workspace(n)
    st = qp.qp_stats(xd, ws)
    assert st.n == n and st.n_nonfinite == 0 and (st.min, st.max) == (-37.0, 40.0)
    # statistics against numpy's pairwise float64 sums, block by block (the tensor is periodic)
    b64 = si.bf16_bits_to_f32(block).astype(np.float64)
    reps, rem = divmod(n, block.size)
    fix = (40.0 - float(si.bf16_bits_to_f32(block[12345:12346])[0])) + (-37.0 - float(si.bf16_bits_to_f32(block[(n - 2) % block.size:(n - 2) % block.size + 1])[0]))
    total = reps * float(b64.sum()) + float(b64[:rem].sum()) + fix
    assert st.mean == pytest.approx(total / n, rel=1e-9, abs=1e-12)
    hist_off = qp.qp_ws_offset(qp.QP_WS_HIST)
    assert int(ws[hist_off:hist_off + 8192].cpu().numpy().view(np.uint32).astype(np.int64).sum()) == n
    for bits in (3, 16):
        print(f"[case] largest tensor: bits={bits}", flush=True)
        res, q = qp.qp_dsaciq_search(xd, st, bits, ws)
        oq = orc.make_qparams(st.mean, res.alpha_star, bits, n)
        assert (q.lo, q.hi, q.scale, q.inv_scale) == (oq.lo, oq.hi, oq.scale, oq.inv_scale)
        packed = qp.alloc_packed(n, bits)
        qp.qp_quant_pack(xd, q, packed)
        y = torch.empty(n, dtype=torch.float32, device="cuda")
        qp.qp_unpack_dequant(packed, q, y)
        torch.cuda.synchronize()
        # sampled windows (multiples of 32 codes, so each is a whole number of packed dwords)
        starts = [0, 32 * 1000003, 32 * (2 ** 26 + 7), (n // 32 - 3000) * 32]
        for s0 in starts:
            s1 = min(n, s0 + 32 * 4000) if s0 != starts[-1] else n
            xw = orc.widen_bf16(h[s0:s1])
            codes = orc.quantize(xw, oq)
            ref = orc.pack(codes, bits)
            got = packed[s0 * bits // 8: s0 * bits // 8 + ref.size].cpu().numpy()
            assert np.array_equal(got, ref), (bits, s0)
            assert np.array_equal(y[s0:s1].cpu().numpy(), orc.dequantize(codes, oq)), (bits, s0)
        assert packed.numel() == 4 * ((n * bits + 31) // 32)
        # the score of the winner on a periodic tensor: periods x (one period's error) + the remainder's + the two
        # changed elements, from the oracle
        def err_of(bits_arr):
            return pairwise_sq_error(orc.widen_bf16(np.ascontiguousarray(bits_arr)), oq)
        e_total = reps * err_of(block) + err_of(block[:rem])
        for i, v in ((12345, 40.0), (n - 2, -37.0)):
            e_total += err_of(si.f32_to_bf16_bits(np.array([v], np.float32))) - err_of(block[i % block.size:i % block.size + 1])
        assert res.mse_star == pytest.approx(e_total / n, rel=1e-9)
        del packed, y


@pytest.mark.timeout(1500)
def test_fp32_tensor_beyond_4_gib(qp):
    """n = 2^30 + 77 fp32 elements (4.3 GB in, byte offsets beyond 2^32): the streaming kernels of statistics,
    search, pack and unpack with 64-bit indexing and a ragged tail.  The tensor is periodic, so the oracle's
    sums over one period give the expected totals."""
    n = 2 ** 30 + 77
    rng = np.random.default_rng(7)
    block = rng.laplace(0.05, 0.6, size=1 << 22).astype(np.float32)
    h = np.tile(block, (n + block.size - 1) // block.size)[:n]
    h[54321] = np.float32(33.0)       # the maximum
    h[n - 3] = np.float32(-29.5)      # the minimum, in the ragged tail
    print("[case] fp32 beyond 4 GiB: upload", flush=True)
    xd = torch.from_numpy(h).cuda()
    ws = qp.alloc_workspace(n)
    st = qp.qp_stats(xd, ws)
    assert st.n == n and st.n_nonfinite == 0 and (st.min, st.max) == (-29.5, 33.0)
    b64 = block.astype(np.float64)
    reps, rem = divmod(n, block.size)
    changed = ((54321, 33.0), (n - 3, -29.5))
    fix = sum(v - float(block[i % block.size]) for i, v in changed)
    total = reps * float(b64.sum()) + float(b64[:rem].sum()) + fix
    assert st.mean == pytest.approx(total / n, rel=1e-9, abs=1e-12)
    dev_block = np.abs(b64 - st.mean)
    mad = reps * float(dev_block.sum()) + float(dev_block[:rem].sum()) + sum(
        abs(v - st.mean) - abs(float(block[i % block.size]) - st.mean) for i, v in changed)
    assert st.mad == pytest.approx(mad / n, rel=1e-9)
    hist_off = qp.qp_ws_offset(qp.QP_WS_HIST)
    assert int(ws[hist_off:hist_off + 8192].cpu().numpy().view(np.uint32).astype(np.int64).sum()) == n
    for bits in (2, 6):
        print(f"[case] fp32 beyond 4 GiB: bits={bits}", flush=True)
        res, q = qp.qp_dsaciq_search(xd, st, bits, ws)
        oq = orc.make_qparams(st.mean, res.alpha_star, bits, n)
        assert (q.lo, q.hi, q.scale, q.inv_scale) == (oq.lo, oq.hi, oq.scale, oq.inv_scale)
        # the winner's score: periods x (one period's error) + the remainder's + the two changed elements
        def err_of(values):
            return pairwise_sq_error(np.ascontiguousarray(values, dtype=np.float32), oq)
        e_total = reps * err_of(block) + err_of(block[:rem]) + sum(
            err_of(np.array([v], np.float32)) - err_of(block[i % block.size:i % block.size + 1]) for i, v in changed)
        assert res.mse_star == pytest.approx(e_total / n, rel=1e-9)
        packed = qp.alloc_packed(n, bits)
        qp.qp_quant_pack(xd, q, packed)
        y = torch.empty(n, dtype=torch.float32, device="cuda")
        qp.qp_unpack_dequant(packed, q, y)
        torch.cuda.synchronize()
        starts = [0, 32 * 1000003, 32 * (2 ** 25 + 11), (n // 32 - 3000) * 32]   # the third lies beyond 2^32 bytes
        for s0 in starts:
            s1 = min(n, s0 + 32 * 4000) if s0 != starts[-1] else n
            codes = orc.quantize(h[s0:s1], oq)
            ref = orc.pack(codes, bits)
            got = packed[s0 * bits // 8: s0 * bits // 8 + ref.size].cpu().numpy()
            assert np.array_equal(got, ref), (bits, s0)
            assert np.array_equal(y[s0:s1].cpu().numpy(), orc.dequantize(codes, oq)), (bits, s0)
        assert packed.numel() == 4 * ((n * bits + 31) // 32)
        del packed, y


# ----------------------------------------------------------------------------- sender path on edge cases, graphs, streams

def check_sender_result(qp, x, bits, ws, packed, t_steps=100, nbins=2048):
    """A finished qp_compress_async call against the oracle: statistics and histogram, the scores of
    all candidates (oracle given the GPU's statistics), the winner, and the packed stream (oracle
    given the GPU's grid)."""
    xf = as_f32(x)
    n = x.size
    st = qp.read_ws(ws, qp.QP_WS_STATS, qp.qp_stats_t)
    rc, ref, hist_ref = orc.stats(xf, nbins=nbins, want_hist=True)
    assert rc == 0 and st.n == ref.n == n and st.n_nonfinite == 0
    assert (st.min, st.max, st.nbins, st.peak_count) == (ref.min, ref.max, nbins, ref.peak_count)
    for f in ("mean", "mad", "abs_mean", "var"):
        a, b = getattr(st, f), getattr(ref, f)
        scale = max(abs(b), ref.abs_mean * 1e-3 if f == "mean" else 0.0)
        # from about 10^6 terms on, the oracle's own term-by-term sums are the less exact side
        assert abs(a - b) <= (REL_STATS if n < (1 << 19) else REL_STATS_FULL) * scale, (f, a, b)
    off = qp.qp_ws_offset(qp.QP_WS_HIST)
    hist = ws[off:off + 4 * nbins].cpu().numpy().view(np.uint32)
    assert np.array_equal(hist, hist_ref[:nbins])
    assert st.b_r == pytest.approx(ref.b_r, rel=1e-14) and st.peak_density == pytest.approx(ref.peak_density, rel=1e-14)
    res = qp.read_ws(ws, qp.QP_WS_RESULT, qp.qp_search_result_t)
    q = qp.read_ws(ws, qp.QP_WS_QPARAMS, qp.qp_qparams_t)
    off = qp.qp_ws_offset(qp.QP_WS_SCORES)
    scores = ws[off:off + 8 * (t_steps + 1)].cpu().numpy().view(np.float64)
    ores, oq, oscores = orc.dsaciq_search(xf, oracle_stats_from(st), bits, t_steps)
    # from about 10^6 terms on, the oracle's term-by-term sum is itself off by ~1e-11: the pairwise sum is the tight check
    tol = REL_SCORE if n < (1 << 19) else REL_SCORE_FULL
    assert np.allclose(scores, oscores, rtol=tol, atol=0.0, equal_nan=True)
    if n >= (1 << 19):
        for j in (0, t_steps // 3, t_steps):
            oqj = orc.make_qparams(st.mean, orc.laplace_F(bits) * (ores.b_e + j * ((ores.b_r - ores.b_e) / t_steps)), bits, n)
            assert scores[j] == pytest.approx(pairwise_sq_error(xf, oqj), rel=REL_SCORE_PAIRWISE)
    assert res.t_steps == t_steps and (res.b_e, res.b_r) == (ores.b_e, ores.b_r)
    if res.j_star != ores.j_star:   # only an exact numerical tie may differ
        assert abs(oscores[res.j_star] - oscores[ores.j_star]) <= 1e-12 * oscores[ores.j_star]
        oq = orc.make_qparams(st.mean, res.alpha_star, bits, n)
    else:
        assert res.alpha_star == pytest.approx(ores.alpha_star, rel=1e-14)
        assert res.mse_star == pytest.approx(ores.mse_star, rel=tol, nan_ok=True)
    assert res.mse_aciq == pytest.approx(ores.mse_aciq, rel=tol, nan_ok=True)
    assert (q.bits, q.n, q.lo, q.hi, q.scale, q.inv_scale) == (bits, n, oq.lo, oq.hi, oq.scale, oq.inv_scale)
    assert np.array_equal(packed.cpu().numpy(), orc.pack(orc.quantize(xf, oracle_q_from(q)), bits))
    return st, res, q


@pytest.mark.parametrize("name,x", si.edge_cases(), ids=[c[0] for c in si.edge_cases()])
def test_sender_path_on_edge_cases(qp, name, x):
    """qp_compress_async on the edge cases, fp32 and bf16: against the oracle, and bit for bit against
    the step-by-step calls (which run the same kernels, with the statistics finalized separately)."""
    for xin in (x, si.f32_to_bf16_bits(x)):
        xd = to_dev(xin)
        n = xin.size
        for bits in (2, 6):
            print(f"[case] sender {name} {xin.dtype} n={n} bits={bits}", flush=True)
            ws = qp.alloc_workspace(n)
            ws.fill_(0xC3)                              # the workspace needs no initialisation
            packed = qp.alloc_packed(n, bits)
            packed.fill_(0x77)
            qp.qp_compress_async(xd, bits, ws, packed)
            torch.cuda.synchronize()
            st, res, q = check_sender_result(qp, xin, bits, ws, packed)
            ws2 = qp.alloc_workspace(n)
            st2 = qp.qp_stats(xd, ws2)
            res2, q2 = qp.qp_dsaciq_search(xd, st2, bits, ws2)
            p2 = qp.alloc_packed(n, bits)
            qp.qp_quant_pack(xd, q2, p2)
            assert bytes(st) == bytes(st2) and bytes(q) == bytes(q2) and torch.equal(packed, p2)
            assert bytes(res) == bytes(res2) or (np.isnan(res2.mse_star) and res.j_star == res2.j_star)


SENDER_CASES = [("C1", None, BITS), ("C5", 151_296, BITS), ("C2", 605_187, (3, 8)), ("C3", 1_048_576, (4, 16)), ("C2", 2_097_152, (4,)),
                    ("C4", 77_773, (2, 6)), ("C5", 999_999, (2, 3)), ("C5", 1_300_001, (4,))]


@pytest.mark.parametrize("name,n,bitset", SENDER_CASES, ids=[f"{c[0]}_{c[1]}" for c in SENDER_CASES])
def test_sender_path_matches_oracle(qp, name, n, bitset):
    """qp_compress_async on small and medium tensors (searched with one candidate per lane): every
    intermediate it leaves in the workspace is checked."""
    x = si.make_config(name, n=n)
    xd = to_dev(x)
    ws = qp.alloc_workspace(x.size)
    qrec = torch.zeros(32, dtype=torch.uint8, device="cuda")
    for bits in bitset:
        print(f"[case] sender {name} n={x.size} bits={bits}", flush=True)
        packed = qp.alloc_packed(x.size, bits)
        qp.qp_compress_async(xd, bits, ws, packed, qparams_out_dev_ptr=qrec.data_ptr())
        torch.cuda.synchronize()
        st, res, q = check_sender_result(qp, x, bits, ws, packed)
        assert bytes(qrec.cpu().numpy().tobytes()) == bytes(q)
        y = torch.empty(x.size, dtype=torch.float32, device="cuda")
        qp.qp_unpack_dequant_dev(packed, bits, qrec.data_ptr(), y)
        oq = oracle_q_from(q)
        assert np.array_equal(y.cpu().numpy(), orc.dequantize(orc.quantize(as_f32(x), oq), oq))


@pytest.mark.parametrize("n", [1, 3, 4, 127, 128, 129, 511, 513, 4095, 4097, 32_768, 65_537, 262_147, 1_048_575, 2_097_151])
def test_sender_path_sizes(qp, n):
    x = si.unit_laplace(n, seed=n) * np.float32(0.7) + np.float32(0.1)
    xd = to_dev(x)
    for bits in (3, 4):
        print(f"[case] sender size n={n} bits={bits}", flush=True)
        ws = qp.alloc_workspace(n)
        ws.fill_(0x3C)
        packed = qp.alloc_packed(n, bits)
        qp.qp_compress_async(xd, bits, ws, packed)
        torch.cuda.synchronize()
        check_sender_result(qp, x, bits, ws, packed)


def test_sender_and_receiver_on_random_sizes(qp):
    """Forty seeded random cases: size log-uniform in [1, 3 M] (so the tile search, the streaming search and, for bf16,
    the value table all occur), fp32 or bf16, any bitwidth, a random location and scale."""
    rng = np.random.default_rng(20221108)
    for case in range(40):
        n = int(np.exp(rng.uniform(0.0, np.log(3.0e6))))
        bits = int(rng.choice(BITS))
        bf16 = bool(rng.integers(0, 2))
        loc, scale = float(rng.normal(0.0, 2.0)), float(np.exp(rng.uniform(np.log(1e-3), np.log(50.0))))
        x32 = (si.unit_laplace(n, seed=1000 + case) * np.float32(scale) + np.float32(loc)).astype(np.float32)
        x = si.f32_to_bf16_bits(x32) if bf16 else x32
        print(f"[case] random #{case}: n={n} bits={bits} bf16={bf16} loc={loc:.3g} scale={scale:.3g}", flush=True)
        xd = to_dev(x)
        ws = qp.alloc_workspace(n)
        ws.fill_(0xC3)
        packed = qp.alloc_packed(n, bits)
        qp.qp_compress_async(xd, bits, ws, packed)
        torch.cuda.synchronize()
        st, res, q = check_sender_result(qp, x, bits, ws, packed)
        y = torch.empty(n, dtype=torch.float32, device="cuda")
        qp.qp_unpack_dequant_dev(packed, bits, ws.data_ptr() + qp.qp_ws_offset(qp.QP_WS_QPARAMS), y)
        oq = oracle_q_from(q)
        assert np.array_equal(y.cpu().numpy(), orc.dequantize(orc.quantize(as_f32(x), oq), oq)), case


def test_sender_path_other_grids(qp):
    x = si.make_config("C2", n=200_003)
    xd = to_dev(x)
    for t, nbins in ((1, 2048), (10, 16), (100, 4096), (255, 100)):
        cfg = qp.qp_default_search_cfg()
        cfg.t_steps, cfg.nbins = t, nbins
        ws = qp.alloc_workspace(x.size, cfg)
        packed = qp.alloc_packed(x.size, 4)
        print(f"[case] sender t={t} nbins={nbins}", flush=True)
        qp.qp_compress_async(xd, 4, ws, packed, cfg=cfg)
        torch.cuda.synchronize()
        check_sender_result(qp, x, 4, ws, packed, t_steps=t, nbins=nbins)


def test_sender_path_is_bit_reproducible(qp):
    x = si.make_config("C1")
    xd = to_dev(x)
    outs = []
    for rep in range(4):
        ws = qp.alloc_workspace(x.size)
        ws.fill_(rep * 37 + 1)
        packed = qp.alloc_packed(x.size, 3)
        qp.qp_compress_async(xd, 3, ws, packed)
        torch.cuda.synchronize()
        off = qp.qp_ws_offset(qp.QP_WS_SCORES)
        outs.append((bytes(qp.read_ws(ws, qp.QP_WS_STATS, qp.qp_stats_t)), bytes(qp.read_ws(ws, qp.QP_WS_RESULT, qp.qp_search_result_t)),
                     ws[off:off + 8 * 101].cpu().numpy().tobytes(), packed.cpu().numpy().tobytes()))
    assert all(o == outs[0] for o in outs[1:])


@pytest.mark.parametrize("kind,n", [("fp32", 700_003), ("fp32", 2_500_003), ("bf16", 1_300_003)],
                         ids=["tile_search", "streaming_search", "value_table"])
def test_sender_and_receiver_replay_from_a_hip_graph(qp, kind, n):
    """The async entry points launch kernels only (no allocation, no memset, no host sync), so they
    capture into a HIP graph; every replay must reproduce the eager result.  One size per search kernel."""
    if kind == "fp32":
        x1, x2 = si.make_config("C2", n=n), si.make_config("C3", n=n)
    else:
        x1 = si.make_config("C5", n=n)
        x2 = si.f32_to_bf16_bits(si.make_config("C3", n=n))
    xin = to_dev(x1).clone()
    ws = qp.alloc_workspace(n)
    packed = qp.alloc_packed(n, 4)
    y = torch.empty(n, dtype=torch.float32, device="cuda")
    qdev = ws.data_ptr() + qp.qp_ws_offset(qp.QP_WS_QPARAMS)

    def run():
        qp.qp_compress_async(xin, 4, ws, packed)
        qp.qp_unpack_dequant_dev(packed, 4, qdev, y)

    def eager(src):
        xin.copy_(to_dev(src))
        run()
        torch.cuda.synchronize()
        return packed.clone(), y.clone(), bytes(qp.read_ws(ws, qp.QP_WS_RESULT, qp.qp_search_result_t))

    ref1, ref2 = eager(x1), eager(x2)
    s = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        run()                                   # warm the stream (and the library's occupancy cache)
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=s):
        run()
    torch.cuda.synchronize()
    for rep, (src, ref) in enumerate(((x1, ref1), (x2, ref2), (x1, ref1), (x2, ref2))):
        xin.copy_(to_dev(src))
        packed.zero_()
        y.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(packed, ref[0]) and torch.equal(y, ref[1]), rep
        assert bytes(qp.read_ws(ws, qp.QP_WS_RESULT, qp.qp_search_result_t)) == ref[2], rep


def test_two_streams_with_their_own_workspaces(qp):
    xa, xb = si.make_config("C2", n=900_001), si.make_config("C3", n=1_100_003)
    da, db = to_dev(xa), to_dev(xb)
    wa, wb = qp.alloc_workspace(xa.size), qp.alloc_workspace(xb.size)
    pa, pb = qp.alloc_packed(xa.size, 3), qp.alloc_packed(xb.size, 8)
    ra_, rb_ = qp.alloc_packed(xa.size, 3), qp.alloc_packed(xb.size, 8)
    qp.qp_compress_async(da, 3, wa, ra_)
    qp.qp_compress_async(db, 8, wb, rb_)
    torch.cuda.synchronize()
    ref = (bytes(qp.read_ws(wa, qp.QP_WS_RESULT, qp.qp_search_result_t)), bytes(qp.read_ws(wb, qp.QP_WS_RESULT, qp.qp_search_result_t)))
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    for _ in range(5):
        pa.zero_(); pb.zero_()
        torch.cuda.synchronize()
        with torch.cuda.stream(sa):
            qp.qp_compress_async(da, 3, wa, pa)
        with torch.cuda.stream(sb):
            qp.qp_compress_async(db, 8, wb, pb)
        torch.cuda.synchronize()
        assert torch.equal(pa, ra_) and torch.equal(pb, rb_)
        assert (bytes(qp.read_ws(wa, qp.QP_WS_RESULT, qp.qp_search_result_t)), bytes(qp.read_ws(wb, qp.QP_WS_RESULT, qp.qp_search_result_t))) == ref


def test_many_tensors_in_flight_match_the_single_calls(qp):
    """qp_compress_many_async: seven tensors of mixed size, dtype and bitwidth (tile search, streaming search, value table)
    over three lanes; every payload and grid record equals what qp_compress_async leaves for that tensor alone, and each
    lane's workspace ends with the records of its last job."""
    specs = [("C2", 700_001, 4), ("C5", 1_300_003, 3), ("C3", 2_500_003, 2), ("C1", None, 8), ("C2", 5, 16), ("C5", 300_001, 6),
             ("C4", 2_200_001, 4)]
    xs = [si.make_config(name, n=n) for name, n, _ in specs]
    ds = [to_dev(x) for x in xs]
    nmax = max(x.size for x in xs)
    ws1 = qp.alloc_workspace(nmax)
    ref = []
    for d, (_, _, bits) in zip(ds, specs):
        pk = qp.alloc_packed(d.numel(), bits)
        qp.qp_compress_async(d, bits, ws1, pk)
        torch.cuda.synchronize()
        ref.append((pk, bytes(qp.read_ws(ws1, qp.QP_WS_QPARAMS, qp.qp_qparams_t)),
                    bytes(qp.read_ws(ws1, qp.QP_WS_RESULT, qp.qp_search_result_t))))
    lanes = [(qp.alloc_workspace(nmax), torch.cuda.Stream()) for _ in range(3)]
    for w, _ in lanes:
        w.fill_(0x77)
    for rep in range(3):
        pks = [qp.alloc_packed(d.numel(), bits) for d, (_, _, bits) in zip(ds, specs)]
        qrecs = torch.zeros(len(specs) * 32, dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()
        jobs = [(d, bits, pk, qrecs.data_ptr() + 32 * k) for k, (d, (_, _, bits), pk) in enumerate(zip(ds, specs, pks))]
        qp.qp_compress_many_async(jobs, lanes)
        torch.cuda.synchronize()
        q_host = qrecs.cpu().numpy().tobytes()
        for k in range(len(specs)):
            assert torch.equal(pks[k], ref[k][0]), (rep, k)
            assert q_host[32 * k:32 * k + 32] == ref[k][1], (rep, k)
        for lane, last in ((0, 6), (1, 4), (2, 5)):
            assert bytes(qp.read_ws(lanes[lane][0], qp.QP_WS_RESULT, qp.qp_search_result_t)) == ref[last][2], (rep, lane)
    # the last jobs of the lanes may leave their grids in the workspace only
    jobs[4] = jobs[4][:3] + (0,)
    jobs[6] = jobs[6][:3] + (0,)
    qp.qp_compress_many_async(jobs, lanes)
    torch.cuda.synchronize()
    assert bytes(qp.read_ws(lanes[0][0], qp.QP_WS_QPARAMS, qp.qp_qparams_t)) == ref[6][1]
    jobs[0] = jobs[0][:3] + (0,)
    with pytest.raises(qp.QuantPipeError):
        qp.qp_compress_many_async(jobs, lanes)


@pytest.mark.timeout(600)
def test_timed_step_spread_over_four_streams(qp):
    """The kind of launch configuration bench.py times (it takes three lanes; four here, so that the lanes carry unequal
    numbers of passes): the six passes of a step over the full C2 tensor handed round-robin to streams, each with its
    own workspace, several steps in flight.  Every payload, output and result record equals what the same pass
    leaves when it runs alone on one stream (whose parity with the oracle the tests above hold)."""
    x = si.make_config("C2")
    n, bits_set = x.size, si.CONFIG_BITS["C2"]
    d = to_dev(x)
    ws = qp.alloc_workspace(n)
    y = torch.empty(n, dtype=torch.float32, device="cuda")
    ref = {}
    for b in bits_set:
        pk = qp.alloc_packed(n, b)
        qp.qp_compress_async(d, b, ws, pk)
        qp.qp_unpack_dequant_dev(pk, b, ws.data_ptr() + qp.qp_ws_offset(qp.QP_WS_QPARAMS), y)
        torch.cuda.synchronize()
        ref[b] = (pk, y.clone(), bytes(qp.read_ws(ws, qp.QP_WS_RESULT, qp.qp_search_result_t)),
                  bytes(qp.read_ws(ws, qp.QP_WS_QPARAMS, qp.qp_qparams_t)))
    lanes = [(torch.cuda.Stream(), qp.alloc_workspace(n)) for _ in range(4)]
    steps = 3
    out = {(s, b): (qp.alloc_packed(n, b), torch.empty(n, dtype=torch.float32, device="cuda")) for s in range(steps) for b in bits_set}
    recs = {}
    torch.cuda.synchronize()
    k = 0
    for s in range(steps):
        for b in bits_set:
            st, w = lanes[k % 4]
            k += 1
            pk, yy = out[(s, b)]
            qp.qp_compress_async(d, b, w, pk, stream=st)
            qp.qp_unpack_dequant_dev(pk, b, w.data_ptr() + qp.qp_ws_offset(qp.QP_WS_QPARAMS), yy, stream=st)
            # the records of this pass, copied out on its stream before the next pass on that stream overwrites them
            with torch.cuda.stream(st):
                recs[(s, b)] = w.clone()
    torch.cuda.synchronize()
    for (s, b), (pk, yy) in out.items():
        assert torch.equal(pk, ref[b][0]), (s, b)
        assert torch.equal(yy, ref[b][1]), (s, b)
        w = recs[(s, b)]
        assert bytes(qp.read_ws(w, qp.QP_WS_RESULT, qp.qp_search_result_t)) == ref[b][2], (s, b)
        assert bytes(qp.read_ws(w, qp.QP_WS_QPARAMS, qp.qp_qparams_t)) == ref[b][3], (s, b)


# ----------------------------------------------------------------------------- histogram-fit reading of Eq. 1

HIST_CASES =[("C1", None), ("C2", 1_234_567), ("C3", 987_653), ("C5", 777_779)]


@pytest.mark.parametrize("name,n", HIST_CASES, ids=[c[0] for c in HIST_CASES])
def test_hist_search_matches_oracle(qp, name, n):
    x = si.make_config(name, n=n)
    xd = to_dev(x)
    ws = qp.alloc_workspace(x.size)
    st = qp.qp_stats(xd, ws)
    off = qp.qp_ws_offset(qp.QP_WS_HIST)
    hist = ws[off:off + 4 * 2048].cpu().numpy().view(np.uint32).copy()
    offs = qp.qp_ws_offset(qp.QP_WS_SCORES)
    for bits, t in ((2, 100), (4, 100), (8, 37)):
        cfg = qp.qp_default_search_cfg()
        cfg.t_steps = t
        res, q = qp.qp_dsaciq_hist_search(bits, ws, cfg=cfg)
        scores = ws[offs:offs + 8 * (t + 1)].cpu().numpy().view(np.float64)
        ores, oq, oscores = orc.hist_search(oracle_stats_from(st), hist, bits, t)
        # the device's exp and libm's may differ in the last place; sums of 2048 terms
        assert np.allclose(scores, oscores, rtol=1e-12, atol=0.0)
        if res.j_star == ores.j_star:
            assert res.alpha_star == pytest.approx(ores.alpha_star, rel=1e-14)
            assert (q.lo, q.hi, q.scale, q.inv_scale, q.bits, q.n) == (oq.lo, oq.hi, oq.scale, oq.inv_scale, bits, x.size)
        else:
            assert abs(oscores[res.j_star] - oscores[ores.j_star]) <= 1e-12 * oscores[ores.j_star]
        assert res.mse_star == pytest.approx(ores.mse_star, rel=1e-12) and res.mse_star <= res.mse_aciq
        assert res.t_steps == t
    # the winner's grid is usable as it is: pack with it straight from the workspace
    packed = qp.alloc_packed(x.size, 8)
    qp.qp_quant_pack_dev(xd, 8, ws.data_ptr() + qp.qp_ws_offset(qp.QP_WS_QPARAMS), packed)
    assert np.array_equal(packed.cpu().numpy(), orc.pack(orc.quantize(as_f32(x), oracle_q_from(q)), 8))


@pytest.mark.parametrize("name", ["constant", "zeros", "two_point", "laplace_n1", "huge_outlier", "large_values"])
def test_hist_search_degenerate_inputs(qp, name):
    x = dict(si.edge_cases())[name]
    xd = to_dev(x)
    ws = qp.alloc_workspace(x.size)
    st = qp.qp_stats(xd, ws)
    off = qp.qp_ws_offset(qp.QP_WS_HIST)
    hist = ws[off:off + 4 * 2048].cpu().numpy().view(np.uint32).copy()
    res, q = qp.qp_dsaciq_hist_search(4, ws)
    ores, oq, oscores = orc.hist_search(oracle_stats_from(st), hist, 4, 100)
    offs = qp.qp_ws_offset(qp.QP_WS_SCORES)
    scores = ws[offs:offs + 8 * 101].cpu().numpy().view(np.float64)
    assert np.allclose(scores, oscores, rtol=1e-12, atol=0.0, equal_nan=True)
    assert res.j_star == ores.j_star
    assert (q.lo, q.hi, q.scale, q.inv_scale) == (oq.lo, oq.hi, oq.scale, oq.inv_scale)


@pytest.mark.parametrize("fill", [0x00, 0xFF, 0x11])
def test_hist_search_on_a_workspace_the_statistics_never_wrote(qp, fill):
    """The histogram-fit search takes its bin count from the record in the workspace.  A record that is not one
    (zeros, all ones, a pattern whose bin count lies far beyond the histogram region) must not be followed out of
    bounds: every score is NaN and the kernel ends normally.  (Whether a result record is written as well depends on
    the ticket word the statistics would have cleared: with a zeroed workspace it is, and keeps plain ACIQ's index.)"""
    ws = qp.alloc_workspace(100_000)
    ws.fill_(fill)
    res, q = qp.qp_dsaciq_hist_search(4, ws)
    offs = qp.qp_ws_offset(qp.QP_WS_SCORES)
    scores = ws[offs:offs + 8 * 101].cpu().numpy().view(np.float64)
    assert np.isnan(scores).all()
    if fill == 0:
        assert res.j_star == 0 and res.t_steps == 100
    # and the workspace is still usable afterwards
    x = si.make_config("C1")
    xd = to_dev(x)
    ws2 = qp.alloc_workspace(x.size)
    ws2.fill_(fill)
    st = qp.qp_stats(xd, ws2)
    res2, q2 = qp.qp_dsaciq_hist_search(4, ws2)
    hist = ws2[qp.qp_ws_offset(qp.QP_WS_HIST):][:4 * 2048].cpu().numpy().view(np.uint32).copy()
    ores, oq, oscores = orc.hist_search(oracle_stats_from(st), hist, 4, 100)
    assert res2.j_star == ores.j_star


@pytest.mark.parametrize("kind", ["constant", "two_point", "ramp_of_all_patterns", "laplace_ragged"])
def test_bf16_value_table_search_edge_cases(qp, kind):
    """Large bf16 tensors are searched through the table of their (at most 65536) distinct values."""
    n = (1 << 20) + 13
    rng = np.random.default_rng(17)
    if kind == "constant":
        x = np.full(n, 0.75, np.float32)
    elif kind == "two_point":
        x = np.where(np.arange(n) % 3 == 0, -1.5, 2.0).astype(np.float32)
    elif kind == "ramp_of_all_patterns":
        # every finite bf16 pattern occurs (about eight times each)
        pats = np.arange(65536, dtype=np.uint32)
        pats = pats[(pats & 0x7F80) != 0x7F80].astype(np.uint16)
        h = np.tile(pats, n // pats.size + 1)[:n]
        x = None
    else:
        x = rng.laplace(0.2, 0.8, size=n).astype(np.float32)
    if x is not None:
        h = si.f32_to_bf16_bits(x)
    xf = orc.widen_bf16(h)
    xd = to_dev(h)
    ws = qp.alloc_workspace(n)
    st = qp.qp_stats(xd, ws)
    offs = qp.qp_ws_offset(qp.QP_WS_SCORES)
    for bits in (2, 8):
        res, q = qp.qp_dsaciq_search(xd, st, bits, ws)
        scores = ws[offs:offs + 8 * 101].cpu().numpy().view(np.float64)
        ores, oq, oscores = orc.dsaciq_search(xf, oracle_stats_from(st), bits, 100)
        assert np.allclose(scores, oscores, rtol=REL_SCORE_FULL, atol=0.0, equal_nan=True)
        F = orc.laplace_F(bits)
        regular = st.mad > 0 and st.b_r > 0 and np.isfinite(st.b_r)   # else the grid collapses onto b_E
        for j in ((0, 100) if regular else ()):
            b = st.mad + j * ((st.b_r - st.mad) / 100)
            oqj = orc.make_qparams(st.mean, F * b, bits, n)
            if np.isfinite(oscores[j]):
                assert scores[j] == pytest.approx(pairwise_sq_error(xf, oqj), rel=REL_SCORE_PAIRWISE, abs=1e-300)
        assert res.j_star == ores.j_star or abs(oscores[res.j_star] - oscores[ores.j_star]) <= 1e-9 * abs(oscores[ores.j_star])
        if res.j_star == ores.j_star:
            assert (q.lo, q.hi, q.scale, q.inv_scale, q.n) == (oq.lo, oq.hi, oq.scale, oq.inv_scale, n)
        assert res.mse_star == pytest.approx(scores[res.j_star] / n, rel=1e-15) or np.isnan(res.mse_star)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("kind", ["constant", "three_values", "hot_value_in_noise"])
def test_bf16_value_table_counters_with_hot_values(qp, kind):
    """Large bf16 tensors whose elements pile onto one or a few values (every lane's increment of the value table
    then hits the same counter, and two of the values differ in sign only): the table's statistics, histogram and
    scores must still be the oracle's."""
    n = (1 << 25) + 13                       # 33.5 M elements
    rng = np.random.default_rng(41)
    if kind == "constant":
        h = si.f32_to_bf16_bits(np.full(n, -0.75, np.float32))
    elif kind == "three_values":             # two of them have the same magnitude and opposite signs
        h = si.f32_to_bf16_bits(np.array([1.5, -1.5, 0.25], np.float32))[rng.integers(0, 3, size=n)]
    else:                                    # 60 % of the elements are one value, the rest Laplace noise
        x = rng.laplace(0.1, 0.5, size=n).astype(np.float32)
        x[rng.random(n) < 0.6] = 0.625
        h = si.f32_to_bf16_bits(x)
    xf = orc.widen_bf16(h)
    xd = to_dev(h)
    ws = qp.alloc_workspace(n)
    st = qp.qp_stats(xd, ws)
    rc, ost, hist_ref = orc.stats(xf, want_hist=True)
    assert (st.n, st.min, st.max, st.peak_count) == (n, ost.min, ost.max, ost.peak_count)
    for f in ("mean", "mad", "abs_mean", "var"):
        assert abs(getattr(st, f) - getattr(ost, f)) <= REL_STATS_FULL * max(abs(getattr(ost, f)), 1e-3 * ost.abs_mean), f
    off = qp.qp_ws_offset(qp.QP_WS_HIST)
    assert np.array_equal(ws[off:off + 8192].cpu().numpy().view(np.uint32), hist_ref[:2048])
    offs = qp.qp_ws_offset(qp.QP_WS_SCORES)
    for bits in (2, 4):
        res, q = qp.qp_dsaciq_search(xd, st, bits, ws)
        scores = ws[offs:offs + 8 * 101].cpu().numpy().view(np.float64)
        ores, oq, oscores = orc.dsaciq_search_threads(xf, oracle_stats_from(st), bits, 100, ORACLE_THREADS)
        assert np.allclose(scores, oscores, rtol=rel_score_sequential(n), atol=0.0, equal_nan=True)
        if check_winner(xf, oracle_stats_from(st), bits, res.j_star, ores):
            assert (q.lo, q.hi, q.scale, q.inv_scale) == (oq.lo, oq.hi, oq.scale, oq.inv_scale)


# ----------------------------------------------------------------------------- variants of the search
# (Gaussian model, ranges intersected with the data's, coarse-to-fine sweep) against their own oracle

VARIANTS = [dict(dist=1), dict(clip=True), dict(stride=10), dict(clip=True, stride=7), dict(dist=1, clip=True, stride=10),
            dict(stride=64), dict(stride=1, clip=True, dist=1)]
# one input per search kernel: tile search (fp32, bf16), streaming search, bf16 value table
VARIANT_INPUTS = [("C3", 300_007), ("C5", 200_003), ("C3", 2_600_011), ("C5", 1_300_001), ("C1", None)]


def variant_cfg(qp, v, t=100):
    cfg = qp.qp_default_search_cfg()
    cfg.t_steps = t
    cfg.dist = v.get("dist", 0)
    cfg.flags = (qp.QP_SEARCH_CLIP_TO_DATA if v.get("clip") else 0) | (qp.QP_SEARCH_COARSE_TO_FINE if v.get("stride", 1) > 1 else 0)
    cfg.coarse_stride = v.get("stride", 1) if v.get("stride", 1) > 1 else 0
    return cfg


def check_variant(qp, xf, st, bits, v, t, ws, res, q):
    n = xf.size
    ores, oq, oscores = orc.dsaciq_search_variant(xf, oracle_stats_from(st), bits, t, dist=v.get("dist", 0),
                                                  clip_to_data=bool(v.get("clip")), stride=v.get("stride", 1))
    off = qp.qp_ws_offset(qp.QP_WS_SCORES)
    scores = ws[off:off + 8 * (t + 1)].cpu().numpy().view(np.float64)
    assert np.array_equal(np.isnan(scores), np.isnan(oscores))            # the same candidates were evaluated
    tol = REL_SCORE if n < (1 << 19) else REL_SCORE_FULL
    assert np.allclose(scores, oscores, rtol=tol, atol=0.0, equal_nan=True)
    assert res.b_e == pytest.approx(ores.b_e, rel=1e-15) and res.b_r == pytest.approx(ores.b_r, rel=1e-15)
    assert res.t_steps == t
    if res.j_star != ores.j_star:   # only an exact numerical tie may differ
        assert abs(oscores[res.j_star] - oscores[ores.j_star]) <= max(1e-12, tol) * oscores[ores.j_star]
    else:
        assert res.alpha_star == pytest.approx(ores.alpha_star, rel=1e-14)
        assert (q.bits, q.n, q.lo, q.hi, q.scale, q.inv_scale) == (bits, n, oq.lo, oq.hi, oq.scale, oq.inv_scale)
        assert res.mse_star == pytest.approx(ores.mse_star, rel=tol)
    assert res.mse_aciq == pytest.approx(ores.mse_aciq, rel=tol)
    return ores


def c2f_offered(x):
    """The coarse-to-fine sweep runs on the tile search for any fp32 tensor; bf16 tensors of 2^20 elements or more go
    through their value table, where it is not offered."""
    return x.size < (1 << 20) if x.dtype == np.uint16 else True


@pytest.mark.parametrize("name,n", VARIANT_INPUTS, ids=[f"{c[0]}_{c[1]}" for c in VARIANT_INPUTS])
def test_search_variants_match_their_oracle(qp, name, n):
    x = si.make_config(name, n=n)
    xf = as_f32(x)
    xd = to_dev(x)
    ws = qp.alloc_workspace(x.size)
    st = qp.qp_stats(xd, ws)
    for v in VARIANTS:
        if v.get("stride", 1) > 1 and not c2f_offered(x):
            continue      # refused by the library there: test_coarse_to_fine_is_refused_on_large_tensors
        for bits in (2, 4):
            print(f"[case] variant {v} {name} n={x.size} bits={bits}", flush=True)
            cfg = variant_cfg(qp, v)
            res, q = qp.qp_dsaciq_search(xd, st, bits, ws, cfg=cfg)
            check_variant(qp, xf, st, bits, v, 100, ws, res, q)


def test_search_variants_other_step_counts_and_strides(qp):
    x = si.make_config("C3", n=150_001)
    xd = to_dev(x)
    for t, stride in ((10, 30), (1, 2), (37, 5), (255, 16), (1000, 10), (100, 2)):
        v = dict(stride=stride, clip=(t % 2 == 1))
        cfg = variant_cfg(qp, v, t)
        ws = qp.alloc_workspace(x.size, cfg)
        st = qp.qp_stats(xd, ws)
        print(f"[case] variant t={t} stride={stride}", flush=True)
        res, q = qp.qp_dsaciq_search(xd, st, 4, ws, cfg=cfg)
        check_variant(qp, x, st, 4, v, t, ws, res, q)


def test_sender_path_with_variants(qp):
    """qp_compress_async with a variant configuration: same bits as the step-by-step calls, payload = the oracle's."""
    for name, n in (("C3", 400_003), ("C3", 2_300_001), ("C5", 1_250_003)):
        x = si.make_config(name, n=n)
        xf = as_f32(x)
        xd = to_dev(x)
        for v in (dict(clip=True), dict(dist=1, stride=10), dict(clip=True, stride=10)):
            if v.get("stride", 1) > 1 and not c2f_offered(x):
                continue
            cfg = variant_cfg(qp, v)
            print(f"[case] sender variant {v} {name} n={n}", flush=True)
            ws = qp.alloc_workspace(n, cfg)
            ws.fill_(0x6B)
            packed = qp.alloc_packed(n, 4)
            qp.qp_compress_async(xd, 4, ws, packed, cfg=cfg)
            torch.cuda.synchronize()
            st = qp.read_ws(ws, qp.QP_WS_STATS, qp.qp_stats_t)
            res = qp.read_ws(ws, qp.QP_WS_RESULT, qp.qp_search_result_t)
            q = qp.read_ws(ws, qp.QP_WS_QPARAMS, qp.qp_qparams_t)
            check_variant(qp, xf, st, 4, v, 100, ws, res, q)
            assert np.array_equal(packed.cpu().numpy(), orc.pack(orc.quantize(xf, oracle_q_from(q)), 4))
            ws2 = qp.alloc_workspace(n, cfg)
            st2 = qp.qp_stats(xd, ws2)
            res2, q2 = qp.qp_dsaciq_search(xd, st2, 4, ws2, cfg=cfg)
            assert bytes(st) == bytes(st2) and bytes(res) == bytes(res2) and bytes(q) == bytes(q2)


def test_clip_to_data_lowers_the_error_of_one_sided_data(qp):
    x = si.make_config("C3", n=1_000_003)
    xd = to_dev(x)
    ws = qp.alloc_workspace(x.size)
    st = qp.qp_stats(xd, ws)
    for bits in (2, 4):
        r0, q0 = qp.qp_dsaciq_search(xd, st, bits, ws)
        r1, q1 = qp.qp_dsaciq_search(xd, st, bits, ws, cfg=variant_cfg(qp, dict(clip=True)))
        assert r1.mse_star < 0.85 * r0.mse_star and q1.lo == np.float32(st.min)


def test_coarse_to_fine_is_refused_on_large_bf16_tensors(qp):
    """bf16 tensors that go through their value table: the coarse-to-fine sweep returns an error before anything is
    launched; the full sweep with the same other settings still runs."""
    x = si.make_config("C5", n=1_300_001)
    xd = to_dev(x)
    ws = qp.alloc_workspace(x.size)
    st = qp.qp_stats(xd, ws)
    with pytest.raises(qp.QuantPipeError) as e:
        qp.qp_dsaciq_search(xd, st, 4, ws, cfg=variant_cfg(qp, dict(stride=10)))
    assert e.value.status == qp.QP_EINVAL
    packed = qp.alloc_packed(x.size, 4)
    with pytest.raises(qp.QuantPipeError):
        qp.qp_compress_async(xd, 4, ws, packed, cfg=variant_cfg(qp, dict(stride=10, clip=True)))
    res, q = qp.qp_dsaciq_search(xd, st, 4, ws, cfg=variant_cfg(qp, dict(clip=True)))
    check_variant(qp, as_f32(x), st, 4, dict(clip=True), 100, ws, res, q)


@pytest.mark.timeout(900)
def test_coarse_to_fine_on_the_full_vit_base_tensor(qp):
    """C2 at full size (9.7 M elements): the sweep runs on the tile search (29 evaluations instead of 101) and finds
    what its oracle finds; on this input that is also the full sweep's winner."""
    x = si.make_config("C2")
    xd = to_dev(x)
    ws = qp.alloc_workspace(x.size)
    st = qp.qp_stats(xd, ws)
    for bits in (2, 4):
        print(f"[case] coarse-to-fine C2 full bits={bits}", flush=True)
        full, qf = qp.qp_dsaciq_search(xd, st, bits, ws)
        res, q = qp.qp_dsaciq_search(xd, st, bits, ws, cfg=variant_cfg(qp, dict(stride=10)))
        check_variant(qp, x, st, bits, dict(stride=10), 100, ws, res, q)
        assert res.j_star == full.j_star and bytes(q) == bytes(qf)


@pytest.mark.skip(reason="the coarse-to-fine sweep on the STREAMING search kernel (k_search_mse with a coarse / fine candidate "
                         "list) faulted the GPU on its only run; the code of that run was never committed, a CPU emulation "
                         "of the launch sequence (blocks one after the other, and blocks of a launch running concurrently "
                         "in shuffled order) is clean under ASan/UBSan, and no cause has been shown.  The library therefore "
                         "refuses such a list in launch_sweep (hipErrorInvalidValue) and runs these sweeps on the tile "
                         "search; this case must not run on a GPU until a cause is shown and fixed")
def test_coarse_to_fine_on_the_streaming_kernel(qp):
    """What would have to pass before the refusal in launch_sweep (csrc/qp_search.hip) may be lifted: with that
    refusal gone and launch_search routing a coarse-to-fine plan on a tensor above the tile search's size limit
    to launch_sweep (coarse list, then fine list), this input (fp32, above 2^21 elements) reaches k_search_mse with
    both lists, in one round (11 and 19 candidates at stride 10) and in several (stride 64: 3 and 127).  As the
    library stands the same calls run on the tile search, so un-skipping alone would not exercise that kernel."""
    x = si.make_config("C3", n=2_600_011)
    assert x.size > (1 << 21)
    xd = to_dev(x)
    ws = qp.alloc_workspace(x.size)
    st = qp.qp_stats(xd, ws)
    for stride in (10, 64):
        for bits in (2, 4):
            res, q = qp.qp_dsaciq_search(xd, st, bits, ws, cfg=variant_cfg(qp, dict(stride=stride)))
            check_variant(qp, x, st, bits, dict(stride=stride), 100, ws, res, q)


# ----------------------------------------------------------------------------- the model chosen per tensor by fit

def gauss_sample(n, seed=21, bf16=False):
    x = (np.random.default_rng(seed).standard_normal(n) * 0.8 + 0.3).astype(np.float32)
    return si.f32_to_bf16_bits(x) if bf16 else x


MODEL_INPUTS = [("C1", lambda: si.make_config("C1")), ("C2", lambda: si.make_config("C2", n=1_234_567)),
                ("C3", lambda: si.make_config("C3", n=987_653)), ("C5_bf16", lambda: si.make_config("C5", n=777_779)),
                ("C5_table", lambda: si.make_config("C5", n=1_300_001)), ("gauss", lambda: gauss_sample(500_003)),
                ("gauss_streaming", lambda: gauss_sample(2_400_007)), ("gauss_table", lambda: gauss_sample(1_500_001, bf16=True)),
                ("constant", lambda: np.full(1000, 1.25, np.float32)), ("one_element", lambda: np.array([0.5], np.float32))]


@pytest.mark.parametrize("name,make", MODEL_INPUTS, ids=[m[0] for m in MODEL_INPUTS])
def test_model_fit_and_search_with_the_chosen_model(qp, name, make):
    """qp_model_fit against the oracle's fit of the same record and histogram; a search with dist = QP_DIST_AUTO
    equals, bit for bit, the search with that model named, and matches the oracle's search under the model the
    oracle chooses; the sender path with QP_DIST_AUTO equals the separate calls."""
    x = make()
    xf = as_f32(x)
    xd = to_dev(x)
    n = x.size
    ws = qp.alloc_workspace(n)
    st = qp.qp_stats(xd, ws)
    hist = ws[qp.qp_ws_offset(qp.QP_WS_HIST):][:4 * 2048].cpu().numpy().view(np.uint32).copy()
    mf = qp.qp_model_fit(ws)
    od, ofl, ofg = orc.model_fit(oracle_stats_from(st), hist)
    print(f"[case] model fit {name} n={n}: laplace {mf.fit_laplace!r} gauss {mf.fit_gauss!r} -> {mf.dist}", flush=True)
    # sums of 2048 terms with the device's exp against libm's
    assert mf.fit_laplace == pytest.approx(ofl, rel=1e-12, nan_ok=True) and mf.fit_gauss == pytest.approx(ofg, rel=1e-12, nan_ok=True)
    if mf.dist != od:      # only a numerical tie between the two fits may be decided differently
        assert abs(ofl - ofg) <= 1e-12 * ofl
    assert mf.dist in (qp.QP_LAPLACE, qp.QP_GAUSS) and mf.reserved == 0
    if name.startswith("gauss"):
        assert mf.dist == qp.QP_GAUSS
    if name in ("C1", "constant", "one_element"):
        assert mf.dist == qp.QP_LAPLACE
    off = qp.qp_ws_offset(qp.QP_WS_SCORES)
    for v in (dict(), dict(clip=True), dict(stride=10)):
        if v.get("stride", 1) > 1 and not c2f_offered(x):
            continue
        auto = variant_cfg(qp, v)
        auto.dist = qp.QP_DIST_AUTO
        named = variant_cfg(qp, dict(v, dist=mf.dist))
        for bits in (2, 8):
            ra, qa = qp.qp_dsaciq_search(xd, st, bits, ws, cfg=auto)
            sa = ws[off:off + 8 * 101].cpu().numpy().tobytes()
            chosen = qp.read_ws(ws, qp.QP_WS_MODEL, qp.qp_model_fit_t)
            assert bytes(chosen) == bytes(mf)
            rn, qn = qp.qp_dsaciq_search(xd, st, bits, ws, cfg=named)
            assert bytes(ra) == bytes(rn) and bytes(qa) == bytes(qn) and sa == ws[off:off + 8 * 101].cpu().numpy().tobytes()
            if mf.dist == od and n > 1:
                check_variant(qp, xf, st, bits, dict(v, dist=od), 100, ws, rn, qn)
    # sender path: statistics, the choice, the search and the pack with nothing returned to the host in between
    auto = qp.qp_default_search_cfg()
    auto.dist = qp.QP_DIST_AUTO
    ws2 = qp.alloc_workspace(n)
    ws2.fill_(0x9E)
    packed = qp.alloc_packed(n, 4)
    qp.qp_compress_async(xd, 4, ws2, packed, cfg=auto)
    torch.cuda.synchronize()
    ra, qa = qp.qp_dsaciq_search(xd, st, 4, ws, cfg=auto)
    assert bytes(qp.read_ws(ws2, qp.QP_WS_MODEL, qp.qp_model_fit_t)) == bytes(mf)
    assert bytes(qp.read_ws(ws2, qp.QP_WS_RESULT, qp.qp_search_result_t)) == bytes(ra)
    assert bytes(qp.read_ws(ws2, qp.QP_WS_QPARAMS, qp.qp_qparams_t)) == bytes(qa)
    assert np.array_equal(packed.cpu().numpy(), orc.pack(orc.quantize(xf, oracle_q_from(qa)), 4))


def test_model_fit_on_a_workspace_the_statistics_never_wrote(qp):
    for fill in (0x00, 0xFF):
        ws = qp.alloc_workspace(50_000)
        ws.fill_(fill)
        mf = qp.qp_model_fit(ws)
        assert np.isnan(mf.fit_laplace) and np.isnan(mf.fit_gauss) and mf.dist == qp.QP_LAPLACE


def test_low_bits_only_policy(qp):
    """QP_SEARCH_LOW_BITS_ONLY (the deployment policy the paper reports: the directed search is active at 2 and 4 bit
    only): above 4 bit the result is plain ACIQ and nothing is scored; at 4 bit and below the search runs as usual."""
    for name, n in (("C1", None), ("C3", 2_600_011), ("C5", 1_300_001)):
        x = si.make_config(name, n=n)
        xf = as_f32(x)
        xd = to_dev(x)
        n_ = x.size
        cfg = qp.qp_default_search_cfg()
        cfg.flags = qp.QP_SEARCH_LOW_BITS_ONLY
        for bits in (16, 8, 6, 4, 2):
            print(f"[case] low-bits-only {name} n={n_} bits={bits}", flush=True)
            ws = qp.alloc_workspace(n_)
            ws.fill_(0x2D)
            packed = qp.alloc_packed(n_, bits)
            qp.qp_compress_async(xd, bits, ws, packed, cfg=cfg)
            torch.cuda.synchronize()
            st = qp.read_ws(ws, qp.QP_WS_STATS, qp.qp_stats_t)
            res = qp.read_ws(ws, qp.QP_WS_RESULT, qp.qp_search_result_t)
            q = qp.read_ws(ws, qp.QP_WS_QPARAMS, qp.qp_qparams_t)
            off = qp.qp_ws_offset(qp.QP_WS_SCORES)
            scores = ws[off:off + 8 * 101].cpu().numpy().view(np.float64)
            if bits > 4:
                alpha = orc.aciq_alpha(oracle_stats_from(st), bits)
                oq = orc.make_qparams(st.mean, alpha, bits, n_)
                assert res.j_star == 0 and res.t_steps == 100 and np.isnan(scores).all()
                assert np.isnan(res.mse_aciq) and np.isnan(res.mse_star)
                assert (res.b_e, res.b_r, res.b_star) == (st.mad, st.b_r, st.mad)
                assert res.alpha_star == pytest.approx(alpha, rel=1e-15)
                assert (q.bits, q.n, q.lo, q.hi, q.scale, q.inv_scale) == (bits, n_, oq.lo, oq.hi, oq.scale, oq.inv_scale)
                assert np.array_equal(packed.cpu().numpy(), orc.pack(orc.quantize(xf, oq), bits))
                # the separate call gives the same record
                st2 = qp.qp_stats(xd, ws)
                res2, q2 = qp.qp_dsaciq_search(xd, st2, bits, ws, cfg=cfg)
                assert bytes(q2) == bytes(q) and res2.j_star == 0 and res2.alpha_star == res.alpha_star
            else:
                check_variant(qp, xf, st, bits, {}, 100, ws, res, q)
                assert np.array_equal(packed.cpu().numpy(), orc.pack(orc.quantize(xf, oracle_q_from(q)), bits))
