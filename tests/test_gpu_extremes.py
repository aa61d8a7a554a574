"""Numerical corner cases on the GPU against the oracle: very large and very small step sizes
(both branches of the softplus evaluation, total and no decay), saturated gates, decay rates over
seven decades, zero inputs."""
import numpy as np
import pytest

from oracle import ss_oracle as orc
from paper_2312_00752_amd import workloads as wl
from tests import util
from tests.test_gpu_bwd import GRADS, ORACLE_NAME

pytestmark = pytest.mark.gpu


def _run(w, io):
    import torch
    from paper_2312_00752_amd import binding as B
    g = util.upload(w)
    nb, nd, nl = w["u"].shape
    nn = w["A"].shape[1]
    ws = torch.empty(B.ss_workspace_bytes(nb, nd, nl, nn, io_dtype=B.SS_BF16 if io == "bf16" else B.SS_F32),
                     dtype=torch.uint8, device="cuda")
    kw = dict(Dskip=g["Dskip"], z=g["z"], delta_bias=g["delta_bias"], delta_softplus=True)
    out, h_last = B.ss_scan_fwd(g["u"], g["delta"], g["A"], g["B"], g["C"], return_last_state=True, workspace=ws, **kw)
    grads = B.ss_scan_bwd(g["dout"], g["u"], g["delta"], g["A"], g["B"], g["C"], ws, **kw)
    torch.cuda.synchronize()
    okw = dict(Dskip=w["Dskip"], z=w["z"], bias=w["delta_bias"], softplus=True)
    ref_f = orc.scan_fwd(w["u"], w["delta"], w["A"], w["B"], w["C"], **okw)
    ref_b = orc.scan_bwd(w["u"], w["delta"], w["A"], w["B"], w["C"], w["dout"], **okw)
    assert torch.isfinite(out.float()).all() and torch.isfinite(h_last).all()
    util.assert_close(out, ref_f["out"], io, "out")
    util.assert_close(h_last, ref_f["h_last"], io, "h_last")
    for k in GRADS:
        if grads.get(k) is not None and k not in ("dh0",):
            assert torch.isfinite(grads[k].float()).all(), k
            util.assert_close(grads[k], ref_b[ORACLE_NAME.get(k, k)], io, k)


@pytest.mark.parametrize("io", ["f32", "bf16"])
def test_step_sizes_from_tiny_to_huge_and_saturated_gates(io):
    rng = np.random.default_rng(1001)
    w = wl.make_scan_inputs(2, 328, 70, 16, io=io, seed=1000)
    rnd = wl.round_to_bf16 if io == "bf16" else (lambda a: a.astype(np.float32))
    # raw step sizes over [-30, 30]: softplus from 1e-13 (series branch) to 30 (identity branch)
    w["delta"] = rnd(rng.uniform(-30.0, 30.0, size=w["delta"].shape).astype(np.float32))
    w["delta_bias"] = np.zeros(70, np.float32)
    # gates from fully closed to fully open
    w["z"] = rnd(rng.uniform(-30.0, 30.0, size=w["z"].shape).astype(np.float32))
    # decay rates over seven decades: exp(dt A) from 1 - 1e-17 down to exact zero (underflow)
    w["A"] = -np.exp(rng.uniform(np.log(1e-4), np.log(1e3), size=(70, 16))).astype(np.float32)
    _run(w, io)


def test_zero_inputs_and_zero_decay():
    w = wl.make_scan_inputs(1, 200, 64, 16, io="f32", seed=1002)
    w["u"][:, ::2] = 0.0          # silent channels
    w["B"][:, :, 50:100] = 0.0    # a stretch with no input at all
    w["A"][:, ::4] = 0.0          # pure accumulators next to decaying states
    _run(w, "f32")
