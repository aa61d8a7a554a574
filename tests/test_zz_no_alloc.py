"""GPU test of ss_scan_fwd_static, the forward entry point that allocates nothing: its scratch is a
fixed array in the library's device image.  Two calls in a row, the second on a smaller problem, each
checked against ss_scan_fwd with a caller-lent workspace (same kernels, so bit-identical) and against
the oracle.  Shapes are chosen so that the scratch is really used: few rows and a long sequence are
split into segments (segment states and step-size sums in the scratch), and B / C are repacked there."""
import numpy as np
import pytest
import torch

from paper_2312_00752_amd import binding as B
from paper_2312_00752_amd import workloads as wl
from tests import util

pytestmark = pytest.mark.gpu


def _run(shape, io, seed):
    nb, nl, nd, nn = shape
    w = wl.make_scan_inputs(nb, nl, nd, nn, io=io, seed=seed)
    g = util.upload(w)
    kw = dict(Dskip=g["Dskip"], z=g["z"], delta_bias=g["delta_bias"], delta_softplus=True)
    need = B.ss_workspace_bytes(nb, nd, nl, nn, for_backward=False, io_dtype=B.SS_BF16 if io == "bf16" else B.SS_F32)
    assert 0 < need <= B.SS_STATIC_SCRATCH_BYTES
    # everything the static call touches exists before it: it must not allocate
    out_s = torch.full_like(g["u"], float("nan"))
    hl_s = torch.full((nb, nd, nn), float("nan"), device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    B.ss_scan_fwd_static(g["u"], g["delta"], g["A"], g["B"], g["C"], out=out_s, h_last=hl_s, **kw)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    out_w, hl_w = B.ss_scan_fwd(g["u"], g["delta"], g["A"], g["B"], g["C"], return_last_state=True,
                                workspace=ws, save_for_bwd=False, **kw)
    torch.cuda.synchronize()
    assert torch.equal(out_s, out_w), "static-scratch call differs from the workspace call"
    assert torch.equal(hl_s, hl_w)
    ref = util.oracle_fwd(w)
    util.assert_close(out_s, ref["out"], io, "out (static scratch)")
    util.assert_close(hl_s, ref["h_last"], io, "h_last (static scratch)")


def test_static_scratch_forward_twice_second_smaller():
    _run((1, 4096, 128, 16), "bf16", 41)   # 2 row groups x 4096 steps: split into segments
    _run((1, 1024, 64, 16), "bf16", 42)    # smaller, right after: stale scratch contents must not matter
    _run((2, 2048, 72, 5), "f32", 43)      # float32 I/O, ragged rows and states


def test_static_scratch_rejects_what_it_cannot_hold():
    p = B.FwdParams()
    p.batch, p.dim, p.seqlen, p.dstate = 1, 256, 1 << 20, 16
    p.io_dtype = B.SS_F32
    fake = torch.empty(16, device="cuda").data_ptr()
    for f in ("u", "delta", "Bmat", "Cmat", "A", "out"):
        setattr(p, f, fake)
    import ctypes
    assert B.lib().ss_scan_fwd_static(ctypes.byref(p), None) == B.SS_ERR_WORKSPACE
    p.seqlen, p.flags = 1024, B.SS_SAVE_FOR_BWD
    assert B.lib().ss_scan_fwd_static(ctypes.byref(p), None) == B.SS_ERR_UNSUPPORTED
