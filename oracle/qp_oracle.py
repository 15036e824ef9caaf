"""ctypes binding of the C oracle (oracle/qp_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  Nothing in the product package imports this, and
this imports nothing from the product package.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

LAPLACE, GAUSS = 0, 1
BITS = (2, 3, 4, 6, 8, 16)


class Stats(C.Structure):
    _fields_ = [("n", C.c_uint64), ("n_nonfinite", C.c_uint64),
                ("mean", C.c_double), ("mad", C.c_double), ("abs_mean", C.c_double),
                ("var", C.c_double), ("min", C.c_double), ("max", C.c_double),
                ("nbins", C.c_uint32), ("peak_count", C.c_uint32),
                ("peak_density", C.c_double), ("b_r", C.c_double)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


class QParams(C.Structure):
    _fields_ = [("bits", C.c_uint32), ("levels", C.c_uint32), ("n", C.c_uint64),
                ("lo", C.c_float), ("hi", C.c_float), ("scale", C.c_float), ("inv_scale", C.c_float)]


class SearchResult(C.Structure):
    _fields_ = [("b_e", C.c_double), ("b_r", C.c_double), ("b_star", C.c_double),
                ("alpha_star", C.c_double), ("mse_aciq", C.c_double), ("mse_star", C.c_double),
                ("j_star", C.c_uint32), ("t_steps", C.c_uint32)]


_lib = None


class Controller(C.Structure):
    _fields_ = [("window", C.c_uint32), ("count", C.c_uint32), ("bits_sum", C.c_double), ("seconds_sum", C.c_double),
                ("s_images", C.c_double), ("r_rate", C.c_double), ("q_cur", C.c_uint32), ("decisions", C.c_uint32)]


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
            _build.build(force=True)
        L = C.CDLL(path)
        fp, u32p, u8p, u16p, dp = (C.POINTER(C.c_float), C.POINTER(C.c_uint32), C.POINTER(C.c_uint8),
                                   C.POINTER(C.c_uint16), C.POINTER(C.c_double))
        L.orc_widen_bf16.argtypes = [u16p, C.c_uint64, fp]
        L.orc_widen_bf16.restype = None
        L.orc_stats.argtypes = [fp, C.c_uint64, C.c_uint32, C.POINTER(Stats), u32p]
        L.orc_stats.restype = C.c_int
        L.orc_lambert_w0.argtypes = [C.c_double]
        L.orc_lambert_w0.restype = C.c_double
        L.orc_laplace_F.argtypes = [C.c_uint32]
        L.orc_laplace_F.restype = C.c_double
        L.orc_gauss_G.argtypes = [C.c_uint32]
        L.orc_gauss_G.restype = C.c_double
        L.orc_aciq_alpha.argtypes = [C.POINTER(Stats), C.c_uint32, C.c_int, dp]
        L.orc_aciq_alpha.restype = C.c_int
        L.orc_make_qparams.argtypes = [C.c_double, C.c_double, C.c_uint32, C.c_uint64, C.POINTER(QParams)]
        L.orc_make_qparams.restype = C.c_int
        L.orc_quant_one.argtypes = [C.c_float, C.POINTER(QParams)]
        L.orc_quant_one.restype = C.c_uint32
        L.orc_dequant_one.argtypes = [C.c_uint32, C.POINTER(QParams)]
        L.orc_dequant_one.restype = C.c_float
        L.orc_quantize.argtypes = [fp, C.c_uint64, C.POINTER(QParams), u32p]
        L.orc_quantize.restype = None
        L.orc_dequantize.argtypes = [u32p, C.c_uint64, C.POINTER(QParams), fp]
        L.orc_dequantize.restype = None
        L.orc_packed_bytes.argtypes = [C.c_uint64, C.c_uint32]
        L.orc_packed_bytes.restype = C.c_uint64
        L.orc_pack.argtypes = [u32p, C.c_uint64, C.c_uint32, u8p, C.c_uint64]
        L.orc_pack.restype = C.c_int
        L.orc_unpack.argtypes = [u8p, C.c_uint64, C.c_uint32, u32p]
        L.orc_unpack.restype = C.c_int
        L.orc_sq_error.argtypes = [fp, C.c_uint64, C.POINTER(QParams)]
        L.orc_sq_error.restype = C.c_double
        L.orc_dsaciq_search.argtypes = [fp, C.c_uint64, C.POINTER(Stats), C.c_uint32, C.c_uint32,
                                        C.POINTER(SearchResult), C.POINTER(QParams), dp]
        L.orc_dsaciq_search.restype = C.c_int
        L.orc_search_candidate.argtypes = [C.POINTER(Stats), C.c_uint32, C.c_uint32, C.c_uint64, C.c_uint32,
                                           C.POINTER(QParams)]
        L.orc_search_candidate.restype = C.c_int
        L.orc_search_pick.argtypes = [C.POINTER(Stats), C.c_uint32, C.c_uint32, C.c_uint64, dp, C.POINTER(SearchResult),
                                      C.POINTER(QParams)]
        L.orc_search_pick.restype = C.c_int
        L.orc_hist_search.argtypes = [C.POINTER(Stats), u32p, C.c_uint32, C.c_uint32, C.POINTER(SearchResult),
                                      C.POINTER(QParams), dp]
        L.orc_hist_search.restype = C.c_int
        L.orc_next_bits.argtypes = [C.c_double, C.c_uint32, C.c_double, C.c_double, C.c_double, C.POINTER(C.c_uint32)]
        L.orc_next_bits.restype = C.c_int
        L.orc_controller_init.argtypes = [C.POINTER(Controller), C.c_uint32, C.c_double, C.c_double, C.c_uint32]
        L.orc_controller_init.restype = C.c_int
        L.orc_controller_update.argtypes = [C.POINTER(Controller), C.c_double, C.c_double, C.POINTER(C.c_uint32)]
        L.orc_controller_update.restype = C.c_int
        L.orc_make_qparams_clipped.argtypes = [C.c_double, C.c_double, C.c_double, C.c_double, C.c_uint32, C.c_uint64,
                                               C.POINTER(QParams)]
        L.orc_make_qparams_clipped.restype = C.c_int
        L.orc_c2f_pick.argtypes = [dp, C.c_uint32, C.c_uint32, u8p]
        L.orc_c2f_pick.restype = C.c_uint32
        L.orc_dsaciq_search_variant.argtypes = [fp, C.c_uint64, C.POINTER(Stats), C.c_uint32, C.c_uint32, C.c_int, C.c_int,
                                                C.c_uint32, C.POINTER(SearchResult), C.POINTER(QParams), dp]
        L.orc_dsaciq_search_variant.restype = C.c_int
        L.orc_model_fit.argtypes = [C.POINTER(Stats), u32p, dp, dp]
        L.orc_model_fit.restype = C.c_int
        _lib = L
    return _lib


def _f32(x):
    a = np.ascontiguousarray(x, dtype=np.float32).reshape(-1)
    return a, a.ctypes.data_as(C.POINTER(C.c_float))


def _u32(x):
    a = np.ascontiguousarray(x, dtype=np.uint32).reshape(-1)
    return a, a.ctypes.data_as(C.POINTER(C.c_uint32))


def widen_bf16(h):
    h = np.ascontiguousarray(h, dtype=np.uint16).reshape(-1)
    out = np.empty(h.size, dtype=np.float32)
    lib().orc_widen_bf16(h.ctypes.data_as(C.POINTER(C.c_uint16)), h.size, out.ctypes.data_as(C.POINTER(C.c_float)))
    return out


def stats(x, nbins=2048, want_hist=False):
    """Returns (status, Stats[, hist]); status 0 ok, 1 non-finite input, 2 bad argument."""
    a, p = _f32(x)
    st = Stats()
    hist = np.zeros(max(nbins, 1), dtype=np.uint32)
    rc = lib().orc_stats(p, a.size, nbins, C.byref(st), hist.ctypes.data_as(C.POINTER(C.c_uint32)))
    return (rc, st, hist) if want_hist else (rc, st)


def lambert_w0(z):
    return lib().orc_lambert_w0(float(z))


def laplace_F(bits):
    return lib().orc_laplace_F(int(bits))


def gauss_G(bits):
    return lib().orc_gauss_G(int(bits))


def aciq_alpha(st, bits, dist=LAPLACE):
    out = C.c_double()
    rc = lib().orc_aciq_alpha(C.byref(st), int(bits), int(dist), C.byref(out))
    if rc:
        raise ValueError("orc_aciq_alpha: bad argument")
    return out.value


def make_qparams(center, alpha, bits, n):
    q = QParams()
    rc = lib().orc_make_qparams(float(center), float(alpha), int(bits), int(n), C.byref(q))
    if rc:
        raise ValueError("orc_make_qparams: bad bitwidth")
    return q


def qparams_from_floats(bits, n, lo, hi, scale, inv_scale):
    """A QParams record holding exactly these floats (e.g. the ones the GPU produced)."""
    q = QParams()
    q.bits, q.levels, q.n = int(bits), (1 << int(bits)) - 1, int(n)
    q.lo, q.hi, q.scale, q.inv_scale = lo, hi, scale, inv_scale
    return q


def quantize(x, q):
    a, p = _f32(x)
    codes = np.empty(a.size, dtype=np.uint32)
    lib().orc_quantize(p, a.size, C.byref(q), codes.ctypes.data_as(C.POINTER(C.c_uint32)))
    return codes


def dequantize(codes, q):
    c, p = _u32(codes)
    y = np.empty(c.size, dtype=np.float32)
    lib().orc_dequantize(p, c.size, C.byref(q), y.ctypes.data_as(C.POINTER(C.c_float)))
    return y


def packed_bytes(n, bits):
    return int(lib().orc_packed_bytes(int(n), int(bits)))


def pack(codes, bits):
    c, p = _u32(codes)
    nb = packed_bytes(c.size, bits)
    if nb == 0 and c.size:
        raise ValueError("bad bitwidth")
    out = np.zeros(nb, dtype=np.uint8)
    rc = lib().orc_pack(p, c.size, int(bits), out.ctypes.data_as(C.POINTER(C.c_uint8)), nb) if c.size else 0
    if rc:
        raise ValueError("orc_pack failed")
    return out


def unpack(buf, n, bits):
    b = np.ascontiguousarray(buf, dtype=np.uint8).reshape(-1)
    codes = np.empty(int(n), dtype=np.uint32)
    rc = lib().orc_unpack(b.ctypes.data_as(C.POINTER(C.c_uint8)), int(n), int(bits),
                          codes.ctypes.data_as(C.POINTER(C.c_uint32)))
    if rc:
        raise ValueError("orc_unpack failed")
    return codes


def sq_error(x, q):
    a, p = _f32(x)
    return lib().orc_sq_error(p, a.size, C.byref(q))


def dsaciq_search(x, st, bits, t_steps=100):
    """Returns (SearchResult, QParams of the winner, scores[t+1])."""
    a, p = _f32(x)
    res, q = SearchResult(), QParams()
    scores = np.zeros(t_steps + 1, dtype=np.float64)
    rc = lib().orc_dsaciq_search(p, a.size, C.byref(st), int(bits), int(t_steps), C.byref(res), C.byref(q),
                                 scores.ctypes.data_as(C.POINTER(C.c_double)))
    if rc:
        raise ValueError("orc_dsaciq_search: bad argument")
    return res, q, scores


def search_candidate(st, bits, t_steps, n, j):
    """The grid of candidate j of the search (what orc_dsaciq_search scores at step j)."""
    q = QParams()
    if lib().orc_search_candidate(C.byref(st), int(bits), int(t_steps), int(n), int(j), C.byref(q)):
        raise ValueError("orc_search_candidate: bad argument")
    return q


def search_pick(st, bits, t_steps, n, scores):
    """The search's decision from all t+1 scores.  Returns (SearchResult, QParams of the winner)."""
    sc = np.ascontiguousarray(scores, dtype=np.float64)
    if sc.size != t_steps + 1:
        raise ValueError("need t_steps + 1 scores")
    res, q = SearchResult(), QParams()
    if lib().orc_search_pick(C.byref(st), int(bits), int(t_steps), int(n), sc.ctypes.data_as(C.POINTER(C.c_double)),
                             C.byref(res), C.byref(q)):
        raise ValueError("orc_search_pick: bad argument")
    return res, q


def dsaciq_search_threads(x, st, bits, t_steps=100, threads=16):
    """orc_dsaciq_search with its candidates spread over host threads: each candidate is scored by the
    same orc_sq_error call, alone and in index order over the tensor (ctypes releases the interpreter
    lock during the call), and orc_search_pick then decides.  Same values as dsaciq_search(), bit for bit;
    the oracle's arithmetic is untouched, only the wall-clock changes."""
    from concurrent.futures import ThreadPoolExecutor
    a, p = _f32(x)
    L = lib()

    def one(j):
        q = search_candidate(st, bits, t_steps, a.size, j)
        return L.orc_sq_error(p, a.size, C.byref(q))

    with ThreadPoolExecutor(max_workers=threads) as ex:
        scores = np.array(list(ex.map(one, range(t_steps + 1))), dtype=np.float64)
    res, q = search_pick(st, bits, t_steps, a.size, scores)
    return res, q, scores


def next_bits(v_bits, q_cur, s_images, r_rate, bandwidth):
    out = C.c_uint32()
    rc = lib().orc_next_bits(float(v_bits), int(q_cur), float(s_images), float(r_rate), float(bandwidth), C.byref(out))
    if rc:
        raise ValueError("orc_next_bits: bad argument")
    return out.value


def hist_search(st, hist, bits, t_steps=100):
    """Histogram-fit reading of Eq. 1.  Returns (SearchResult, QParams of the winner, scores[t+1])."""
    h, p = _u32(hist)
    if h.size < st.nbins:
        raise ValueError("histogram shorter than st.nbins")
    res, q = SearchResult(), QParams()
    scores = np.zeros(t_steps + 1, dtype=np.float64)
    rc = lib().orc_hist_search(C.byref(st), p, int(bits), int(t_steps), C.byref(res), C.byref(q),
                               scores.ctypes.data_as(C.POINTER(C.c_double)))
    if rc:
        raise ValueError("orc_hist_search: bad argument")
    return res, q, scores


# ---- variants of the directed search (not the paper's method; see the C source) -------------------

LAPLACE, GAUSS = 0, 1


def make_qparams_clipped(center, alpha, data_min, data_max, bits, n):
    q = QParams()
    rc = lib().orc_make_qparams_clipped(float(center), float(alpha), float(data_min), float(data_max), int(bits), int(n),
                                        C.byref(q))
    if rc:
        raise ValueError("orc_make_qparams_clipped: bad bitwidth")
    return q


def c2f_pick(scores, stride):
    """(index a coarse-to-fine sweep with this stride picks from a full score table, mask of the entries it reads)."""
    sc = np.ascontiguousarray(scores, dtype=np.float64)
    ev = np.zeros(sc.size, dtype=np.uint8)
    j = lib().orc_c2f_pick(sc.ctypes.data_as(C.POINTER(C.c_double)), sc.size - 1, int(stride),
                           ev.ctypes.data_as(C.POINTER(C.c_uint8)))
    return int(j), ev.astype(bool)


def dsaciq_search_variant(x, st, bits, t_steps=100, dist=LAPLACE, clip_to_data=False, stride=1):
    """Returns (SearchResult, QParams of the winner, scores[t+1] with NaN where nothing was evaluated)."""
    a, p = _f32(x)
    res, q = SearchResult(), QParams()
    scores = np.zeros(t_steps + 1, dtype=np.float64)
    rc = lib().orc_dsaciq_search_variant(p, a.size, C.byref(st), int(bits), int(t_steps), int(dist), int(bool(clip_to_data)),
                                         int(stride), C.byref(res), C.byref(q), scores.ctypes.data_as(C.POINTER(C.c_double)))
    if rc:
        raise ValueError("orc_dsaciq_search_variant: bad argument")
    return res, q, scores


def model_fit(st, hist):
    """Which model the histogram fits better.  Returns (LAPLACE or GAUSS, fit_laplace, fit_gauss)."""
    h, p = _u32(hist)
    if h.size < st.nbins:
        raise ValueError("histogram shorter than st.nbins")
    fl, fg = C.c_double(), C.c_double()
    d = lib().orc_model_fit(C.byref(st), p, C.byref(fl), C.byref(fg))
    return d, fl.value, fg.value


# ---- adaptive PDA controller (window averages feeding Eq. 2) --------------------------------------

def controller(window, s_images, r_rate, q_start=32):
    c = Controller()
    if lib().orc_controller_init(C.byref(c), int(window), float(s_images), float(r_rate), int(q_start)):
        raise ValueError("orc_controller_init: bad argument")
    return c


def controller_update(c, payload_bits, seconds):
    q = C.c_uint32()
    if lib().orc_controller_update(C.byref(c), float(payload_bits), float(seconds), C.byref(q)):
        raise ValueError("orc_controller_update: bad argument")
    return q.value
