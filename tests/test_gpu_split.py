"""Few rows and a long sequence: the library splits L across workgroups and stitches the
segments with a carry pass.  Parity against the oracle, with and without the scratch."""
import numpy as np
import pytest

from paper_2312_00752_amd import workloads as wl
from tests import util
from tests.test_gpu_bwd import GRADS, ORACLE_NAME

pytestmark = pytest.mark.gpu


def _ws(nbytes):
    import torch
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")


@pytest.mark.parametrize("io,batch,seqlen,dim,dstate", [
    ("f32", 1, 4096, 64, 16),     # 8 segments of 512
    ("bf16", 2, 6144, 100, 16),   # ragged row tile
    ("f32", 1, 4100, 40, 16),     # 8-aligned ragged tail in the last segment
    ("bf16", 1, 4099, 70, 8),     # element-wise path, padded states
    ("f32", 3, 2048, 30, 16),     # shortest sequence that is split
])
def test_split_sequence_forward_and_backward(io, batch, seqlen, dim, dstate):
    import torch
    from paper_2312_00752_amd import binding as B
    w = wl.make_scan_inputs(batch, seqlen, dim, dstate, io=io, seed=200 + seqlen % 97)
    rng = np.random.default_rng(201)
    w["h0"] = rng.normal(size=(batch, dim, dstate)).astype(np.float32)
    w["dh_last"] = rng.normal(size=(batch, dim, dstate)).astype(np.float32)
    code = B.SS_BF16 if io == "bf16" else B.SS_F32
    assert B.ss_workspace_bytes(batch, dim, seqlen, dstate, for_backward=False, io_dtype=code) > 0, \
        "this shape is meant to be split"
    g = util.upload(w)
    kw = dict(Dskip=g["Dskip"], z=g["z"], delta_bias=g["delta_bias"], h0=g["h0"], delta_softplus=True)
    ref_f, ref_b = util.oracle_fwd(w), util.oracle_bwd(w)
    # plain forward: unsplit (no scratch) and split (scratch lent) agree with the oracle
    o1, h1 = B.ss_scan_fwd(g["u"], g["delta"], g["A"], g["B"], g["C"], return_last_state=True, **kw)
    ws0 = _ws(B.ss_workspace_bytes(batch, dim, seqlen, dstate, for_backward=False, io_dtype=code))
    o2, h2 = B.ss_scan_fwd(g["u"], g["delta"], g["A"], g["B"], g["C"], return_last_state=True,
                           workspace=ws0, save_for_bwd=False, **kw)
    torch.cuda.synchronize()
    for o, h, tag in ((o1, h1, "unsplit"), (o2, h2, "split")):
        util.assert_close(o, ref_f["out"], io, "out " + tag)
        util.assert_close(h, ref_f["h_last"], io, "h_last " + tag)
    # training path
    ws = _ws(B.ss_workspace_bytes(batch, dim, seqlen, dstate, io_dtype=code))
    o3, h3 = B.ss_scan_fwd(g["u"], g["delta"], g["A"], g["B"], g["C"], return_last_state=True,
                           workspace=ws, **kw)
    grads = B.ss_scan_bwd(g["dout"], g["u"], g["delta"], g["A"], g["B"], g["C"], ws,
                          dh_last=g["dh_last"], want_dh0=True, **kw)
    torch.cuda.synchronize()
    util.assert_close(o3, ref_f["out"], io, "out (save)")
    util.assert_close(h3, ref_f["h_last"], io, "h_last (save)")
    for k in GRADS:
        util.assert_close(grads[k], ref_b[ORACLE_NAME.get(k, k)], io, k)
