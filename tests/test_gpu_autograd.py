"""The torch.autograd front-ends (marshalling only) against the oracle, and a check that every
output element is really written (outputs pre-filled with NaN)."""
import numpy as np
import pytest

from oracle import inner_oracle as inn
from paper_2312_00752_amd import workloads as wl
from tests import util

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("io", ["f32", "bf16"])
def test_selective_scan_autograd(io):
    import torch
    from paper_2312_00752_amd.autograd import selective_scan
    w = wl.make_scan_inputs(2, 300, 72, 16, io=io, seed=61)
    rng = np.random.default_rng(62)
    w["h0"] = rng.normal(size=(2, 72, 16)).astype(np.float32)
    w["dh_last"] = rng.normal(size=(2, 72, 16)).astype(np.float32)
    g = util.upload(w)
    leaves = {k: g[k].clone().requires_grad_(True) for k in ("u", "delta", "A", "B", "C", "Dskip", "z", "delta_bias", "h0")}
    out, h_last = selective_scan(leaves["u"], leaves["delta"], leaves["A"], leaves["B"], leaves["C"], leaves["Dskip"],
                                 leaves["z"], leaves["delta_bias"], leaves["h0"], delta_softplus=True,
                                 return_last_state=True)
    loss = (out.float() * g["dout"].float()).sum() + (h_last * g["dh_last"]).sum()
    loss.backward()
    torch.cuda.synchronize()
    ref_f, ref_b = util.oracle_fwd(w), util.oracle_bwd(w)
    util.assert_close(out, ref_f["out"], io, "out")
    util.assert_close(h_last, ref_f["h_last"], io, "h_last")
    names = {"u": "du", "delta": "ddelta", "A": "dA", "B": "dB", "C": "dC", "Dskip": "dD", "z": "dz",
             "delta_bias": "dbias", "h0": "dh0"}
    for k, oname in names.items():
        assert leaves[k].grad is not None and leaves[k].grad.dtype == leaves[k].dtype, k
        util.assert_close(leaves[k].grad, ref_b[oname], io, "grad of " + k)


def test_layer_autograd():
    import torch
    from paper_2312_00752_amd.autograd import selective_ssm_layer
    w = wl.make_layer_inputs(2, 264, 96, 16, io="bf16", seed=63, rank=6)
    names = ("x", "z", "conv_w", "conv_b", "W_x", "W_dt", "dt_bias", "A", "Dskip")
    t = {k: torch.from_numpy(w[k]).cuda() for k in names + ("dout",)}
    for k in ("x", "z", "W_x", "W_dt", "dout"):
        t[k] = t[k].to(torch.bfloat16)
    leaves = {k: t[k].clone().requires_grad_(True) for k in names}
    out = selective_ssm_layer(*[leaves[k] for k in names])
    (out.float() * t["dout"].float()).sum().backward()
    torch.cuda.synchronize()
    rnd = lambda a: wl.round_to_bf16(a).astype(np.float64)
    kw = {k: w[k] for k in names}
    ref = inn.inner_fwd(rnd=rnd, **kw)
    rg = inn.inner_bwd(dout=w["dout"], rnd=rnd, **kw)
    util.assert_close(out, ref["out"], "bf16", "out", exact_inputs=False)
    gnames = {"x": "dx", "z": "dz", "conv_w": "dconv_w", "conv_b": "dconv_b", "W_x": "dW_x", "W_dt": "dW_dt",
              "dt_bias": "ddt_bias", "A": "dA", "Dskip": "dD"}
    for k, oname in gnames.items():
        util.assert_close(leaves[k].grad, rg[oname], "bf16", "grad of " + k, exact_inputs=False)


@pytest.mark.parametrize("io,seqlen", [("bf16", 2048 + 24), ("f32", 333), ("bf16", 4096)])
def test_every_output_element_is_written(io, seqlen):
    """Outputs start as NaN; after the calls no NaN may be left (ragged tails, split sequences included)."""
    import torch
    from paper_2312_00752_amd import binding as B
    w = wl.make_scan_inputs(2, seqlen, 70, 16, io=io, seed=64)
    g = util.upload(w)
    code = B.SS_BF16 if io == "bf16" else B.SS_F32
    ws = torch.empty(B.ss_workspace_bytes(2, 70, seqlen, 16, io_dtype=code), dtype=torch.uint8, device="cuda")
    ws.fill_(0xff)                       # NaN patterns in every float the library might read before writing
    nan_like = lambda t: torch.full_like(t, float("nan"))
    out = nan_like(g["u"])
    h_last = torch.full((2, 70, 16), float("nan"), device="cuda")
    kw = dict(Dskip=g["Dskip"], z=g["z"], delta_bias=g["delta_bias"], delta_softplus=True)
    B.ss_scan_fwd(g["u"], g["delta"], g["A"], g["B"], g["C"], out=out, h_last=h_last, workspace=ws, **kw)
    assert not torch.isnan(out.float()).any() and not torch.isnan(h_last).any()
    grads = B.ss_scan_bwd(g["dout"], g["u"], g["delta"], g["A"], g["B"], g["C"], ws, want_dh0=True, **kw)
    ref = util.oracle_bwd(w)
    for k, v in grads.items():
        if v is not None:
            assert not torch.isnan(v.float()).any(), k
    util.assert_close(grads["du"], ref["du"], io, "du")
    # convolution
    c = wl.make_conv_inputs(2, 70, seqlen, 4, io, seed=65)
    tio = torch.bfloat16 if io == "bf16" else torch.float32
    x = torch.from_numpy(c["x"]).cuda().to(tio)
    cw, cb = torch.from_numpy(c["w"]).cuda(), torch.from_numpy(c["bias"]).cuda()
    o = nan_like(x)
    B.ss_conv_fwd(x, cw, cb, out=o)
    assert not torch.isnan(o.float()).any()
