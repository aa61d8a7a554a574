"""Parity at the full sizes of the five workloads, in the launch configuration bench.py
times (needs an MI355X; the oracle runs on the machine's host cores and takes seconds)."""
import gc

import numpy as np
import pytest

from paper_2312_00752_amd import workloads as wl
from tests import util
from tests.test_gpu_bwd import GRADS, ORACLE_NAME

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", wl.CONFIG_ORDER)
def test_full_size_forward_and_backward(name):
    import torch
    from paper_2312_00752_amd import binding as B
    w = wl.make_config(name)
    nb, nl, nd, nn = w["shape"]
    io = w["io"]
    g = util.upload(w)
    ws = torch.empty(B.ss_workspace_bytes(nb, nd, nl, nn, io_dtype=B.SS_BF16 if io == "bf16" else B.SS_F32),
                     dtype=torch.uint8, device="cuda")
    kw = dict(Dskip=g["Dskip"], z=g["z"], delta_bias=g["delta_bias"], delta_softplus=True)
    out, h_last = B.ss_scan_fwd(g["u"], g["delta"], g["A"], g["B"], g["C"], return_last_state=True,
                                workspace=ws, **kw)
    grads = B.ss_scan_bwd(g["dout"], g["u"], g["delta"], g["A"], g["B"], g["C"], ws, want_dh0=True, **kw)
    torch.cuda.synchronize()
    del g, ws
    errs = {}
    ref = util.oracle_fwd(w)
    errs["out"] = util.assert_close(out, ref["out"], io, "out")
    errs["h_last"] = util.assert_close(h_last, ref["h_last"], io, "h_last")
    del ref, out, h_last
    gc.collect()
    ref = util.oracle_bwd(w)
    for k in GRADS:
        errs[k] = util.assert_close(grads[k], ref[ORACLE_NAME.get(k, k)], io, k)
        grads[k] = None
    print(name, {k: "%.1e" % v for k, v in errs.items()})
