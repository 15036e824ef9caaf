"""ctypes binding of include/quantpipe.h: same names, argument marshalling only.

torch is used for device memory and streams: tensors give `data_ptr()`, the current torch
stream gives the hipStream_t.  torch is imported before the library is loaded so that the
library binds to the HIP runtime already in the process.
"""
from __future__ import annotations

import ctypes as C
import os

import torch  # noqa: F401  (must precede CDLL: one HIP runtime per process)

__all__ = [
    "QP_OK", "QP_EINVAL", "QP_ENOSPC", "QP_EHIP", "QP_ENONFINITE", "QP_F32", "QP_BF16", "QP_LAPLACE", "QP_GAUSS", "QP_DIST_AUTO", "QP_WS_MODEL", "qp_model_fit_t", "qp_model_fit", "qp_model_fit_async", "qp_job_t", "qp_lane_t",
    "QP_SEARCH_CLIP_TO_DATA", "QP_SEARCH_COARSE_TO_FINE", "QP_SEARCH_LOW_BITS_ONLY",
    "QP_WS_STATS", "QP_WS_RESULT", "QP_WS_QPARAMS", "QP_WS_HIST", "QP_WS_CANDS", "QP_WS_SCORES",
    "qp_stats_t", "qp_qparams_t", "qp_search_cfg_t", "qp_search_result_t", "qp_controller_t", "QuantPipeError", "BITS",
    "lib", "qp_packed_bytes", "qp_workspace_bytes", "qp_ws_offset", "qp_default_search_cfg", "qp_stats",
    "qp_stats_async", "qp_aciq_alpha", "qp_aciq_constant", "qp_make_qparams", "qp_make_qparams_clipped", "qp_dsaciq_search",
    "qp_dsaciq_search_async", "qp_dsaciq_hist_search", "qp_dsaciq_hist_search_async", "qp_quant_pack", "qp_quant_pack_dev", "qp_unpack_dequant", "qp_unpack_dequant_dev",
    "qp_compress_async", "qp_compress_many_async", "qp_compress_noalloc", "qp_next_bits", "qp_controller_init", "qp_controller_update", "qp_strerror", "alloc_workspace", "alloc_packed", "dtype_of", "read_ws",
]

QP_OK, QP_EINVAL, QP_ENOSPC, QP_EHIP, QP_ENONFINITE = 0, -1, -2, -3, -4
QP_F32, QP_BF16 = 0, 1
QP_LAPLACE, QP_GAUSS, QP_DIST_AUTO = 0, 1, 2
QP_SEARCH_CLIP_TO_DATA, QP_SEARCH_COARSE_TO_FINE, QP_SEARCH_LOW_BITS_ONLY = 1, 2, 4
QP_WS_STATS, QP_WS_RESULT, QP_WS_QPARAMS, QP_WS_HIST, QP_WS_CANDS, QP_WS_SCORES, QP_WS_MODEL = range(7)
BITS = (2, 3, 4, 6, 8, 16)

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libquantpipe.so")


class qp_stats_t(C.Structure):
    _fields_ = [("n", C.c_uint64), ("n_nonfinite", C.c_uint64), ("mean", C.c_double), ("mad", C.c_double),
                ("abs_mean", C.c_double), ("var", C.c_double), ("min", C.c_double), ("max", C.c_double),
                ("nbins", C.c_uint32), ("peak_count", C.c_uint32), ("peak_density", C.c_double),
                ("b_r", C.c_double)]


class qp_qparams_t(C.Structure):
    _fields_ = [("bits", C.c_uint32), ("reserved", C.c_uint32), ("n", C.c_uint64), ("lo", C.c_float),
                ("hi", C.c_float), ("scale", C.c_float), ("inv_scale", C.c_float)]


class qp_search_cfg_t(C.Structure):
    _fields_ = [("t_steps", C.c_uint32), ("cands_per_round", C.c_uint32), ("nbins", C.c_uint32),
                ("dist", C.c_uint32), ("flags", C.c_uint32), ("coarse_stride", C.c_uint32)]


class qp_controller_t(C.Structure):
    _fields_ = [("window", C.c_uint32), ("count", C.c_uint32), ("bits_sum", C.c_double), ("seconds_sum", C.c_double),
                ("s_images", C.c_double), ("r_images_per_s", C.c_double), ("q_cur", C.c_uint32), ("decisions", C.c_uint32)]


class qp_search_result_t(C.Structure):
    _fields_ = [("b_e", C.c_double), ("b_r", C.c_double), ("b_star", C.c_double), ("alpha_star", C.c_double),
                ("mse_aciq", C.c_double), ("mse_star", C.c_double), ("j_star", C.c_uint32),
                ("t_steps", C.c_uint32)]


class qp_model_fit_t(C.Structure):
    _fields_ = [("fit_laplace", C.c_double), ("fit_gauss", C.c_double), ("dist", C.c_uint32), ("reserved", C.c_uint32)]


class qp_job_t(C.Structure):
    _fields_ = [("x_dev", C.c_void_p), ("n", C.c_uint64), ("dtype", C.c_uint32), ("bits", C.c_uint32),
                ("packed_dev", C.c_void_p), ("packed_bytes", C.c_uint64), ("qparams_out_dev", C.c_void_p)]


class qp_lane_t(C.Structure):
    _fields_ = [("ws_dev", C.c_void_p), ("ws_bytes", C.c_size_t), ("stream", C.c_void_p)]


class QuantPipeError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {qp_strerror(status)} ({status})")


_lib = None


def lib():
    """The loaded C-ABI library.  Raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2211_04515_amd.build` "
                              "(or __graft_entry__.build()); there is no CPU fallback")
        L = C.CDLL(LIB_PATH)
        vp, u64, u32, sz, i32 = C.c_void_p, C.c_uint64, C.c_uint32, C.c_size_t, C.c_int
        sig = {
            "qp_packed_bytes": (sz, [u64, u32]),
            "qp_workspace_bytes": (sz, [u64, C.POINTER(qp_search_cfg_t)]),
            "qp_ws_offset": (sz, [i32]),
            "qp_default_search_cfg": (None, [C.POINTER(qp_search_cfg_t)]),
            "qp_stats": (i32, [vp, u64, i32, u32, vp, sz, vp, C.POINTER(qp_stats_t)]),
            "qp_stats_async": (i32, [vp, u64, i32, u32, vp, sz, vp]),
            "qp_aciq_alpha": (i32, [C.POINTER(qp_stats_t), u32, i32, C.POINTER(C.c_double)]),
            "qp_aciq_constant": (C.c_double, [u32, i32]),
            "qp_make_qparams": (i32, [C.c_double, C.c_double, u32, u64, C.POINTER(qp_qparams_t)]),
            "qp_make_qparams_clipped": (i32, [C.c_double, C.c_double, C.c_double, C.c_double, u32, u64,
                                              C.POINTER(qp_qparams_t)]),
            "qp_dsaciq_search": (i32, [vp, u64, i32, C.POINTER(qp_stats_t), u32, C.POINTER(qp_search_cfg_t), vp, sz,
                                       vp, C.POINTER(qp_search_result_t), C.POINTER(qp_qparams_t)]),
            "qp_dsaciq_search_async": (i32, [vp, u64, i32, u32, C.POINTER(qp_search_cfg_t), vp, sz, vp]),
            "qp_model_fit": (i32, [vp, sz, vp, C.POINTER(qp_model_fit_t)]),
            "qp_model_fit_async": (i32, [vp, sz, vp]),
            "qp_dsaciq_hist_search": (i32, [u32, C.POINTER(qp_search_cfg_t), vp, sz, vp, C.POINTER(qp_search_result_t),
                                            C.POINTER(qp_qparams_t)]),
            "qp_dsaciq_hist_search_async": (i32, [u32, C.POINTER(qp_search_cfg_t), vp, sz, vp]),
            "qp_quant_pack": (i32, [vp, u64, i32, C.POINTER(qp_qparams_t), vp, sz, vp]),
            "qp_quant_pack_dev": (i32, [vp, u64, i32, u32, vp, vp, sz, vp]),
            "qp_unpack_dequant": (i32, [vp, sz, C.POINTER(qp_qparams_t), vp, u64, vp]),
            "qp_unpack_dequant_dev": (i32, [vp, sz, u32, vp, vp, u64, vp]),
            "qp_compress_async": (i32, [vp, u64, i32, u32, C.POINTER(qp_search_cfg_t), vp, sz, vp, sz, vp, vp]),
            "qp_compress_noalloc": (i32, [vp, u64, i32, u32, C.POINTER(qp_search_cfg_t), vp, sz, vp, vp]),
            "qp_compress_many_async": (i32, [C.POINTER(qp_job_t), u32, C.POINTER(qp_search_cfg_t), C.POINTER(qp_lane_t), u32]),
            "qp_next_bits": (i32, [C.c_double, u32, C.c_double, C.c_double, C.c_double, C.POINTER(u32)]),
            "qp_controller_init": (i32, [C.POINTER(qp_controller_t), u32, C.c_double, C.c_double, u32]),
            "qp_controller_update": (i32, [C.POINTER(qp_controller_t), C.c_double, C.c_double, C.POINTER(u32)]),
            "qp_strerror": (C.c_char_p, [i32]),
        }
        for name, (res, args) in sig.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


EXPORTS = ("qp_packed_bytes", "qp_workspace_bytes", "qp_ws_offset", "qp_default_search_cfg", "qp_stats",
           "qp_stats_async", "qp_aciq_alpha", "qp_aciq_constant", "qp_make_qparams", "qp_make_qparams_clipped", "qp_dsaciq_search",
           "qp_dsaciq_search_async", "qp_model_fit", "qp_model_fit_async", "qp_dsaciq_hist_search", "qp_dsaciq_hist_search_async", "qp_quant_pack", "qp_quant_pack_dev", "qp_unpack_dequant",
           "qp_unpack_dequant_dev", "qp_compress_async", "qp_compress_many_async", "qp_compress_noalloc", "qp_next_bits", "qp_controller_init", "qp_controller_update",
           "qp_strerror")


# ---- marshalling helpers ------------------------------------------------------------------

def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def dtype_of(t: "torch.Tensor") -> int:
    if t.dtype == torch.float32:
        return QP_F32
    if t.dtype == torch.bfloat16:
        return QP_BF16
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def _dev(t: "torch.Tensor"):
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    return C.c_void_p(t.data_ptr())


def _cfgp(cfg):
    return C.byref(cfg) if cfg is not None else None


def _check(status: int, what: str, allow=()):
    if status != QP_OK and status not in allow:
        raise QuantPipeError(status, what)
    return status


def alloc_workspace(n: int, cfg=None, device="cuda") -> "torch.Tensor":
    nb = qp_workspace_bytes(n, cfg)
    if nb == 0:
        raise QuantPipeError(QP_EINVAL, "qp_workspace_bytes")
    return torch.empty(nb, dtype=torch.uint8, device=device)


def alloc_packed(n: int, bits: int, device="cuda") -> "torch.Tensor":
    nb = qp_packed_bytes(n, bits)
    if nb == 0:
        raise QuantPipeError(QP_EINVAL, "qp_packed_bytes")
    return torch.empty(nb, dtype=torch.uint8, device=device)


def read_ws(ws: "torch.Tensor", region: int, ctype):
    """Copy a fixed-size record out of the workspace (synchronises the current stream)."""
    off = qp_ws_offset(region)
    raw = ws[off:off + C.sizeof(ctype)].cpu().numpy().tobytes()
    return ctype.from_buffer_copy(raw)


# ---- the entry points, names as in quantpipe.h --------------------------------------------

def qp_strerror(status: int) -> str:
    return lib().qp_strerror(int(status)).decode()


def qp_packed_bytes(n: int, bits: int) -> int:
    return int(lib().qp_packed_bytes(int(n), int(bits)))


def qp_workspace_bytes(n: int, cfg=None) -> int:
    return int(lib().qp_workspace_bytes(int(n), _cfgp(cfg)))


def qp_ws_offset(region: int) -> int:
    return int(lib().qp_ws_offset(int(region)))


def qp_default_search_cfg() -> qp_search_cfg_t:
    cfg = qp_search_cfg_t()
    lib().qp_default_search_cfg(C.byref(cfg))
    return cfg


def qp_stats(x, ws, nbins: int = 2048, stream=None, allow_nonfinite: bool = False) -> qp_stats_t:
    out = qp_stats_t()
    st = lib().qp_stats(_dev(x), x.numel(), dtype_of(x), int(nbins), _dev(ws), ws.numel(), _stream(stream),
                        C.byref(out))
    _check(st, "qp_stats", allow=(QP_ENONFINITE,) if allow_nonfinite else ())
    return out


def qp_stats_async(x, ws, nbins: int = 2048, stream=None) -> None:
    _check(lib().qp_stats_async(_dev(x), x.numel(), dtype_of(x), int(nbins), _dev(ws), ws.numel(), _stream(stream)),
           "qp_stats_async")


def qp_aciq_alpha(stats: qp_stats_t, bits: int, dist: int = QP_LAPLACE) -> float:
    out = C.c_double()
    _check(lib().qp_aciq_alpha(C.byref(stats), int(bits), int(dist), C.byref(out)), "qp_aciq_alpha")
    return out.value


def qp_aciq_constant(bits: int, dist: int = QP_LAPLACE) -> float:
    return float(lib().qp_aciq_constant(int(bits), int(dist)))


def qp_make_qparams(center: float, alpha: float, bits: int, n: int) -> qp_qparams_t:
    q = qp_qparams_t()
    _check(lib().qp_make_qparams(float(center), float(alpha), int(bits), int(n), C.byref(q)), "qp_make_qparams")
    return q


def qp_make_qparams_clipped(center: float, alpha: float, data_min: float, data_max: float, bits: int, n: int) -> qp_qparams_t:
    q = qp_qparams_t()
    _check(lib().qp_make_qparams_clipped(float(center), float(alpha), float(data_min), float(data_max), int(bits), int(n),
                                         C.byref(q)), "qp_make_qparams_clipped")
    return q


def qp_dsaciq_search(x, stats: qp_stats_t, bits: int, ws, cfg=None, stream=None):
    """Returns (qp_search_result_t, qp_qparams_t of the winner)."""
    res, q = qp_search_result_t(), qp_qparams_t()
    _check(lib().qp_dsaciq_search(_dev(x), x.numel(), dtype_of(x), C.byref(stats), int(bits), _cfgp(cfg), _dev(ws),
                                  ws.numel(), _stream(stream), C.byref(res), C.byref(q)), "qp_dsaciq_search")
    return res, q


def qp_dsaciq_search_async(x, bits: int, ws, cfg=None, stream=None) -> None:
    _check(lib().qp_dsaciq_search_async(_dev(x), x.numel(), dtype_of(x), int(bits), _cfgp(cfg), _dev(ws), ws.numel(),
                                        _stream(stream)), "qp_dsaciq_search_async")


def qp_quant_pack(x, qparams: qp_qparams_t, packed, stream=None) -> None:
    _check(lib().qp_quant_pack(_dev(x), x.numel(), dtype_of(x), C.byref(qparams), _dev(packed),
                               packed.numel() * packed.element_size(), _stream(stream)), "qp_quant_pack")


def qp_quant_pack_dev(x, bits: int, qparams_dev_ptr: int, packed, stream=None) -> None:
    _check(lib().qp_quant_pack_dev(_dev(x), x.numel(), dtype_of(x), int(bits), C.c_void_p(qparams_dev_ptr),
                                   _dev(packed), packed.numel() * packed.element_size(), _stream(stream)),
           "qp_quant_pack_dev")


def qp_unpack_dequant(packed, qparams: qp_qparams_t, y, stream=None) -> None:
    if y.dtype != torch.float32:
        raise TypeError("y must be float32")
    _check(lib().qp_unpack_dequant(_dev(packed), packed.numel() * packed.element_size(), C.byref(qparams), _dev(y),
                                   y.numel(), _stream(stream)), "qp_unpack_dequant")


def qp_unpack_dequant_dev(packed, bits: int, qparams_dev_ptr: int, y, stream=None) -> None:
    if y.dtype != torch.float32:
        raise TypeError("y must be float32")
    _check(lib().qp_unpack_dequant_dev(_dev(packed), packed.numel() * packed.element_size(), int(bits),
                                       C.c_void_p(qparams_dev_ptr), _dev(y), y.numel(), _stream(stream)),
           "qp_unpack_dequant_dev")


def qp_compress_async(x, bits: int, ws, packed, qparams_out_dev_ptr: int = 0, cfg=None, stream=None) -> None:
    _check(lib().qp_compress_async(_dev(x), x.numel(), dtype_of(x), int(bits), _cfgp(cfg), _dev(ws), ws.numel(),
                                   _dev(packed), packed.numel() * packed.element_size(),
                                   C.c_void_p(qparams_out_dev_ptr) if qparams_out_dev_ptr else None,
                                   _stream(stream)), "qp_compress_async")


def qp_compress_many_async(jobs, lanes, cfg=None) -> None:
    """jobs: sequence of (x, bits, packed, qparams_out_dev_ptr or 0); lanes: sequence of (workspace, stream)."""
    ja = (qp_job_t * len(jobs))()
    for k, (x, bits, packed, qptr) in enumerate(jobs):
        ja[k] = qp_job_t(x.data_ptr(), x.numel(), dtype_of(x), int(bits), packed.data_ptr(),
                         packed.numel() * packed.element_size(), qptr or None)
    la = (qp_lane_t * len(lanes))()
    for k, (ws, stream) in enumerate(lanes):
        la[k] = qp_lane_t(ws.data_ptr(), ws.numel(), _stream(stream).value)
    _check(lib().qp_compress_many_async(ja, len(jobs), _cfgp(cfg), la, len(lanes)), "qp_compress_many_async")


def qp_compress_noalloc(x, bits: int, packed, qparams_out_dev_ptr: int, cfg=None, stream=None) -> None:
    _check(lib().qp_compress_noalloc(_dev(x), x.numel(), dtype_of(x), int(bits), _cfgp(cfg), _dev(packed),
                                     packed.numel() * packed.element_size(), C.c_void_p(qparams_out_dev_ptr),
                                     _stream(stream)), "qp_compress_noalloc")


def qp_next_bits(v_bits: float, q_cur: int, s_images: float, r_images_per_s: float, bandwidth_bits_per_s: float) -> int:
    out = C.c_uint32()
    _check(lib().qp_next_bits(float(v_bits), int(q_cur), float(s_images), float(r_images_per_s),
                              float(bandwidth_bits_per_s), C.byref(out)), "qp_next_bits")
    return out.value


def qp_controller_init(window: int, s_images: float, r_images_per_s: float, q_start: int = 32) -> qp_controller_t:
    c = qp_controller_t()
    _check(lib().qp_controller_init(C.byref(c), int(window), float(s_images), float(r_images_per_s), int(q_start)),
           "qp_controller_init")
    return c


def qp_controller_update(c: qp_controller_t, payload_bits: float, seconds: float) -> int:
    out = C.c_uint32()
    _check(lib().qp_controller_update(C.byref(c), float(payload_bits), float(seconds), C.byref(out)), "qp_controller_update")
    return out.value


def qp_model_fit(ws, stream=None) -> qp_model_fit_t:
    """Which model (Laplace or Gaussian) the statistics and histogram left in ws fit better."""
    out = qp_model_fit_t()
    _check(lib().qp_model_fit(_dev(ws), ws.numel(), _stream(stream), C.byref(out)), "qp_model_fit")
    return out


def qp_model_fit_async(ws, stream=None) -> None:
    _check(lib().qp_model_fit_async(_dev(ws), ws.numel(), _stream(stream)), "qp_model_fit_async")


def qp_dsaciq_hist_search(bits: int, ws, cfg=None, stream=None):
    """Histogram-fit reading of Eq. 1 on the statistics left in ws.  Returns (result, qparams)."""
    res, q = qp_search_result_t(), qp_qparams_t()
    _check(lib().qp_dsaciq_hist_search(int(bits), _cfgp(cfg), _dev(ws), ws.numel(), _stream(stream), C.byref(res),
                                       C.byref(q)), "qp_dsaciq_hist_search")
    return res, q


def qp_dsaciq_hist_search_async(bits: int, ws, cfg=None, stream=None) -> None:
    _check(lib().qp_dsaciq_hist_search_async(int(bits), _cfgp(cfg), _dev(ws), ws.numel(), _stream(stream)),
           "qp_dsaciq_hist_search_async")
