"""The sender path for callers that cannot allocate (qp_compress_noalloc: the workspace is a static
device array inside the library) against qp_compress_async with a caller-owned workspace: same packed
stream and same winner's record, bit for bit, on calls in a row whose inputs shrink (the array keeps
the previous call's contents), for each of the search kernels; and the payload against the oracle.
Runs last in the suite and also alone in a fresh process (the array's address is looked up on the
first call)."""
import ctypes as C

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


@pytest.fixture(scope="module")
def qp():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2211_04515_amd as m
    m.lib()
    return m


def to_dev(x):
    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16).copy()).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()


def both_paths(qp, x, bits, cfg=None):
    """(packed, record) of the no-alloc entry point and of qp_compress_async on the same input."""
    xd = to_dev(x)
    n = x.size
    p_static = qp.alloc_packed(n, bits)
    p_static.fill_(0x5C)
    q_static = torch.zeros(32, dtype=torch.uint8, device="cuda")
    qp.qp_compress_noalloc(xd, bits, p_static, q_static.data_ptr(), cfg=cfg)
    ws = qp.alloc_workspace(n, cfg)
    p_ws = qp.alloc_packed(n, bits)
    q_ws = torch.zeros(32, dtype=torch.uint8, device="cuda")
    qp.qp_compress_async(xd, bits, ws, p_ws, qparams_out_dev_ptr=q_ws.data_ptr(), cfg=cfg)
    torch.cuda.synchronize()
    return p_static, q_static, p_ws, q_ws


# in this order: every call but the first finds the leftovers of a larger input in the array
CALLS = [("C2", 2_500_003, 4),      # streaming search
         ("C3", 700_001, 2),        # tile search, smaller
         ("C5", 1_300_003, 3),      # bf16 value table
         ("C5", 300_011, 8),        # bf16 below the value table's threshold
         ("C1", None, 4),           # one image's activations
         ("C1", 1_001, 16),
         ("C4", 5, 6)]


def test_no_alloc_entry_point_matches_the_workspace_one(qp):
    for name, n, bits in CALLS:
        x = si.make_config(name, n=n)
        print(f"[case] no-alloc {name} n={x.size} bits={bits}", flush=True)
        p_static, q_static, p_ws, q_ws = both_paths(qp, x, bits)
        assert torch.equal(q_static, q_ws), (name, n, bits)
        assert torch.equal(p_static, p_ws), (name, n, bits)
        # and the payload is the oracle's for that grid
        q = qp.qp_qparams_t.from_buffer_copy(q_static.cpu().numpy().tobytes())
        assert (q.bits, q.n) == (bits, x.size)
        xf = orc.widen_bf16(x) if x.dtype == np.uint16 else x
        oq = orc.qparams_from_floats(q.bits, q.n, q.lo, q.hi, q.scale, q.inv_scale)
        assert np.array_equal(p_static.cpu().numpy(), orc.pack(orc.quantize(xf, oq), bits))


def test_no_alloc_entry_point_with_a_search_configuration(qp):
    x = si.make_config("C3", n=400_003)
    cfg = qp.qp_default_search_cfg()
    cfg.t_steps, cfg.flags, cfg.dist = 127, qp.QP_SEARCH_CLIP_TO_DATA, qp.QP_GAUSS
    p_static, q_static, p_ws, q_ws = both_paths(qp, x, 4, cfg)
    assert torch.equal(q_static, q_ws) and torch.equal(p_static, p_ws)


def test_no_alloc_entry_point_rejects_what_it_cannot_hold(qp):
    x = si.make_config("C1")
    xd = to_dev(x)
    packed = qp.alloc_packed(x.size, 4)
    rec = torch.zeros(32, dtype=torch.uint8, device="cuda")
    cfg = qp.qp_default_search_cfg()
    cfg.t_steps = 128                      # one more than the static workspace is sized for
    with pytest.raises(qp.QuantPipeError) as e:
        qp.qp_compress_noalloc(xd, 4, packed, rec.data_ptr(), cfg=cfg)
    assert e.value.status == qp.QP_ENOSPC
    L = qp.lib()
    vp = C.c_void_p
    assert L.qp_compress_noalloc(vp(xd.data_ptr()), x.size, 0, 4, None, vp(packed.data_ptr()), packed.numel(), None, None) == qp.QP_EINVAL
    assert L.qp_compress_noalloc(vp(xd.data_ptr()), x.size, 0, 5, None, vp(packed.data_ptr()), packed.numel(), vp(rec.data_ptr()), None) == qp.QP_EINVAL
    assert L.qp_compress_noalloc(vp(xd.data_ptr()), x.size, 0, 4, None, vp(packed.data_ptr()), 8, vp(rec.data_ptr()), None) == qp.QP_ENOSPC
    assert L.qp_compress_noalloc(vp(xd.data_ptr()), 0, 0, 4, None, vp(packed.data_ptr()), packed.numel(), vp(rec.data_ptr()), None) == qp.QP_EINVAL


def test_no_alloc_entry_point_replays_from_a_hip_graph(qp):
    """Callers under graph capture are whom the entry point is for: after one call outside the capture (the array's
    address is looked up then) it captures, and every replay reproduces the eager result, with the program's own
    eager work between the replays."""
    n = 600_011
    x1, x2 = si.make_config("C2", n=n), si.make_config("C3", n=n)
    xin = to_dev(x1).clone()
    packed = qp.alloc_packed(n, 3)
    rec = torch.zeros(32, dtype=torch.uint8, device="cuda")

    def eager(src):
        xin.copy_(to_dev(src))
        qp.qp_compress_noalloc(xin, 3, packed, rec.data_ptr())
        torch.cuda.synchronize()
        return packed.clone(), rec.clone()

    ref1, ref2 = eager(x1), eager(x2)
    s = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        qp.qp_compress_noalloc(xin, 3, packed, rec.data_ptr())
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=s):
        qp.qp_compress_noalloc(xin, 3, packed, rec.data_ptr())
    torch.cuda.synchronize()
    for rep, (src, ref) in enumerate(((x1, ref1), (x2, ref2), (x1, ref1))):
        xin.copy_(to_dev(src))
        packed.zero_()
        rec.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(packed, ref[0]) and torch.equal(rec, ref[1]), rep
