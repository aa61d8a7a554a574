"""The exact zero-order-hold B-bar of Eq. 4 on the GPU (SS_EXACT_ZOH_B), against the oracle."""
import numpy as np
import pytest
from scipy.special import expit

from oracle import ss_oracle as orc
from paper_2312_00752_amd import workloads as wl
from tests import util
from tests.test_gpu_bwd import GRADS, ORACLE_NAME

pytestmark = pytest.mark.gpu


def _workload(io, batch, seqlen, dim, dstate, seed):
    w = wl.make_scan_inputs(batch, seqlen, dim, dstate, io=io, seed=seed)
    rng = np.random.default_rng(seed + 1)
    # decay rates over five decades, so that dt*A covers both the series and the direct branch,
    # and a few exact zeros (phi = dt there)
    A = -np.exp(rng.uniform(np.log(1e-3), np.log(30.0), size=(dim, dstate)))
    A[rng.random(size=A.shape) < 0.05] = 0.0
    w["A"] = A.astype(np.float32)
    w["h0"] = rng.normal(size=(batch, dim, dstate)).astype(np.float32)
    w["dh_last"] = rng.normal(size=(batch, dim, dstate)).astype(np.float32)
    return w


@pytest.mark.parametrize("io,batch,seqlen,dim,dstate", [
    ("f32", 2, 160, 70, 16), ("bf16", 2, 264, 100, 16), ("f32", 1, 77, 20, 5),
    ("bf16", 3, 203, 65, 13), ("f32", 1, 4096, 64, 16),
])
def test_exact_zoh_forward_and_backward(io, batch, seqlen, dim, dstate):
    import torch
    from paper_2312_00752_amd import binding as B
    w = _workload(io, batch, seqlen, dim, dstate, seed=300 + seqlen)
    g = util.upload(w)
    code = B.SS_BF16 if io == "bf16" else B.SS_F32
    ws = torch.empty(B.ss_workspace_bytes(batch, dim, seqlen, dstate, io_dtype=code), dtype=torch.uint8, device="cuda")
    kw = dict(Dskip=g["Dskip"], z=g["z"], delta_bias=g["delta_bias"], h0=g["h0"], delta_softplus=True,
              exact_zoh=True)
    out, h_last = B.ss_scan_fwd(g["u"], g["delta"], g["A"], g["B"], g["C"], return_last_state=True,
                                workspace=ws, **kw)
    grads = B.ss_scan_bwd(g["dout"], g["u"], g["delta"], g["A"], g["B"], g["C"], ws,
                          dh_last=g["dh_last"], want_dh0=True, **kw)
    torch.cuda.synchronize()
    okw = dict(Dskip=w["Dskip"], z=w["z"], bias=w["delta_bias"], h0=w["h0"], softplus=True, exact_zoh=True)
    ref_f = orc.scan_fwd(w["u"], w["delta"], w["A"], w["B"], w["C"], **okw)
    ref_b = orc.scan_bwd(w["u"], w["delta"], w["A"], w["B"], w["C"], w["dout"], dh_last=w["dh_last"], **okw)
    util.assert_close(out, ref_f["out"], io, "out")
    util.assert_close(h_last, ref_f["h_last"], io, "h_last")
    for k in GRADS:
        util.assert_close(grads[k], ref_b[ORACLE_NAME.get(k, k)], io, k)
    # and it really is a different operator from the first-order rule
    plain = orc.scan_fwd(w["u"], w["delta"], w["A"], w["B"], w["C"], Dskip=w["Dskip"], z=w["z"],
                         bias=w["delta_bias"], h0=w["h0"], softplus=True)
    assert util.rel_err(out, plain["out"]) > 2 * util.TOL[io]


def test_theorem1_gated_recurrence_on_the_gpu():
    """N=1, A=-1, B=C=1, softplus, exact ZOH: h_t = (1-g_t) h_{t-1} + g_t x_t with g = sigmoid(r)."""
    import torch
    from paper_2312_00752_amd import binding as B
    rng = np.random.default_rng(310)
    L, D = 96, 3
    r = (rng.normal(size=(1, D, L)) * 1.5).astype(np.float32)
    x = rng.normal(size=(1, D, L)).astype(np.float32)
    ones = torch.ones(1, 1, L, device="cuda")
    out, _ = B.ss_scan_fwd(torch.from_numpy(x).cuda(), torch.from_numpy(r).cuda(),
                           -torch.ones(D, 1, device="cuda"), ones, ones, delta_softplus=True, exact_zoh=True)
    torch.cuda.synchronize()
    gate = expit(r.astype(np.float64))
    h = np.zeros((1, D))
    want = np.empty((1, D, L))
    for t in range(L):
        h = (1 - gate[..., t]) * h + gate[..., t] * x[..., t]
        want[..., t] = h
    util.assert_close(out, want, "f32", "gated recurrence")


@pytest.mark.parametrize("dstate", [5, 16])
def test_exact_zoh_step(dstate):
    import torch
    from paper_2312_00752_amd import binding as B
    s = wl.make_step_inputs(4, 67, dstate, 6, io="f32", seed=320)
    rng = np.random.default_rng(321)
    A = -np.exp(rng.uniform(np.log(1e-3), np.log(30.0), size=(67, dstate)))
    A[0, 0] = 0.0
    A = A.astype(np.float32)
    h_ref = rng.normal(size=(4, 67, dstate)).astype(np.float32)
    h = torch.from_numpy(h_ref.copy()).cuda()
    h_ref = h_ref.astype(np.float64)
    up = lambda a: torch.from_numpy(a).cuda()
    for t in range(6):
        o = B.ss_step(h, up(s["u"][t]), up(s["delta"][t]), up(A), up(s["B"][t]), up(s["C"][t]),
                      Dskip=up(s["Dskip"]), z_t=up(s["z"][t]), delta_bias=up(s["delta_bias"]),
                      delta_softplus=True, exact_zoh=True)
        o_ref, h_ref = orc.step(h_ref, s["u"][t], s["delta"][t], A, s["B"][t], s["C"][t], Dskip=s["Dskip"],
                                z_t=s["z"][t], bias=s["delta_bias"], softplus=True, exact_zoh=True)
        torch.cuda.synchronize()
        util.assert_close(o, o_ref, "f32", "out_t")
        util.assert_close(h, h_ref, "f32", "h")
