"""More than 16 states: the library handles them 16 at a time in passes that add up (forward,
backward, step, split sequences, time-invariant B / C, the layer), against the oracle."""
import numpy as np
import pytest

from oracle import inner_oracle as inn
from oracle import ss_oracle as orc
from paper_2312_00752_amd import workloads as wl
from tests import util
from tests.test_gpu_bwd import GRADS, ORACLE_NAME

pytestmark = pytest.mark.gpu


def _workload(io, batch, seqlen, dim, dstate, seed):
    w = wl.make_scan_inputs(batch, seqlen, dim, dstate, io=io, seed=seed)
    rng = np.random.default_rng(seed + 3)
    # decay rates spread over the states (the S4D-real ramp -(n+1) would make states past 16 die at once)
    w["A"] = -np.exp(rng.uniform(np.log(0.02), np.log(8.0), size=(dim, dstate))).astype(np.float32)
    # keep the output O(1): C scaled by 1/sqrt(N/16)
    w["C"] = (w["C"] * np.float32(4.0 / np.sqrt(dstate))).astype(np.float32)
    if io == "bf16":
        w["C"] = wl.round_to_bf16(w["C"])
    w["h0"] = rng.normal(size=(batch, dim, dstate)).astype(np.float32)
    w["dh_last"] = rng.normal(size=(batch, dim, dstate)).astype(np.float32)
    return w


@pytest.mark.parametrize("io,batch,seqlen,dim,dstate,zoh,gate", [
    ("f32", 2, 160, 70, 32, False, True), ("bf16", 2, 264, 100, 64, False, True), ("f32", 1, 77, 20, 17, False, True),
    ("bf16", 3, 203, 65, 40, True, True), ("f32", 1, 4096, 64, 48, False, True), ("f32", 2, 200, 64, 33, False, False),
    ("bf16", 1, 512, 128, 256, False, True),
])
def test_many_states_forward_and_backward(io, batch, seqlen, dim, dstate, zoh, gate):
    import torch
    from paper_2312_00752_amd import binding as B
    w = _workload(io, batch, seqlen, dim, dstate, 700 + seqlen)
    g = util.upload(w)
    code = B.SS_BF16 if io == "bf16" else B.SS_F32
    ws = torch.empty(B.ss_workspace_bytes(batch, dim, seqlen, dstate, io_dtype=code, has_z=gate), dtype=torch.uint8, device="cuda")
    kw = dict(Dskip=g["Dskip"], z=g["z"] if gate else None, delta_bias=g["delta_bias"], h0=g["h0"], delta_softplus=True,
              exact_zoh=zoh)
    out, h_last = B.ss_scan_fwd(g["u"], g["delta"], g["A"], g["B"], g["C"], return_last_state=True, workspace=ws, **kw)
    grads = B.ss_scan_bwd(g["dout"], g["u"], g["delta"], g["A"], g["B"], g["C"], ws, dh_last=g["dh_last"], want_dh0=True, **kw)
    torch.cuda.synchronize()
    okw = dict(Dskip=w["Dskip"], z=w["z"] if gate else None, bias=w["delta_bias"], h0=w["h0"], softplus=True, exact_zoh=zoh)
    ref_f = orc.scan_fwd(w["u"], w["delta"], w["A"], w["B"], w["C"], **okw)
    ref_b = orc.scan_bwd(w["u"], w["delta"], w["A"], w["B"], w["C"], w["dout"], dh_last=w["dh_last"], **okw)
    # the io-dtype tensors that every pass of 16 states adds to (pre-gate y, du, ddelta) are rounded once per pass
    fl = util.ELEM_FLOOR_ROUNDED if io == "bf16" else None
    util.assert_close(out, ref_f["out"], io, "out", elem_floor=fl)
    util.assert_close(h_last, ref_f["h_last"], io, "h_last")
    for k in GRADS:
        if grads[k] is not None:
            util.assert_close(grads[k], ref_b[ORACLE_NAME.get(k, k)], io, k, elem_floor=fl if k in ("du", "ddelta", "dz") else None)
    # plain forward (nothing kept for backward): with a gate the workspace carries the running sum
    ws0 = torch.empty(max(256, B.ss_workspace_bytes(batch, dim, seqlen, dstate, False, code, gate)), dtype=torch.uint8, device="cuda")
    out2, _ = B.ss_scan_fwd(g["u"], g["delta"], g["A"], g["B"], g["C"], workspace=ws0, save_for_bwd=False, **kw)
    util.assert_close(out2, ref_f["out"], io, "plain forward out", elem_floor=fl)
    if gate:
        with pytest.raises(B.SsError):
            B.ss_scan_fwd(g["u"], g["delta"], g["A"], g["B"], g["C"], **kw)


def test_many_states_time_invariant_bc():
    import torch
    from paper_2312_00752_amd import binding as B
    w = _workload("f32", 2, 300, 66, 24, 801)
    rng = np.random.default_rng(802)
    w["B"] = rng.normal(size=(66, 24)).astype(np.float32)
    w["C"] = (rng.normal(size=(66, 24)) * 0.5).astype(np.float32)
    t = lambda a: torch.from_numpy(a).cuda()
    g = util.upload({k: v for k, v in w.items() if k not in ("B", "C")} | {"B": None, "C": None})
    g["B"], g["C"] = t(w["B"]), t(w["C"])
    ws = torch.empty(B.ss_workspace_bytes(2, 66, 300, 24, io_dtype=B.SS_F32, b_fixed=True, c_fixed=True), dtype=torch.uint8, device="cuda")
    kw = dict(Dskip=g["Dskip"], z=g["z"], delta_bias=g["delta_bias"], delta_softplus=True)
    out, _ = B.ss_scan_fwd(g["u"], g["delta"], g["A"], g["B"], g["C"], workspace=ws, **kw)
    grads = B.ss_scan_bwd(g["dout"], g["u"], g["delta"], g["A"], g["B"], g["C"], ws, **kw)
    torch.cuda.synchronize()
    okw = dict(Dskip=w["Dskip"], z=w["z"], bias=w["delta_bias"], softplus=True)
    util.assert_close(out, orc.scan_fwd(w["u"], w["delta"], w["A"], w["B"], w["C"], **okw)["out"], "f32", "out")
    ref_b = orc.scan_bwd(w["u"], w["delta"], w["A"], w["B"], w["C"], w["dout"], **okw)
    for k in ("du", "ddelta", "dz", "dB", "dC", "dA", "dD", "ddelta_bias"):
        util.assert_close(grads[k], ref_b[ORACLE_NAME.get(k, k)], "f32", k)


@pytest.mark.parametrize("dstate", [20, 64])
def test_many_states_step(dstate):
    import torch
    from paper_2312_00752_amd import binding as B
    nb, nd, tokens = 3, 40, 7
    s = wl.make_step_inputs(nb, nd, dstate, tokens, io="bf16", seed=33)
    rng = np.random.default_rng(34)
    A = -np.exp(rng.uniform(np.log(0.02), np.log(8.0), size=(nd, dstate))).astype(np.float32)
    bf = torch.bfloat16
    g = {k: torch.from_numpy(s[k]).cuda().to(bf) for k in ("u", "delta", "z", "B", "C")}
    At, Dk, bias = torch.from_numpy(A).cuda(), torch.from_numpy(s["Dskip"]).cuda(), torch.from_numpy(s["delta_bias"]).cuda()
    h = torch.zeros(nb, nd, dstate, device="cuda")
    href = np.zeros((nb, nd, dstate))
    for i in range(tokens):
        o = B.ss_step(h, g["u"][i], g["delta"][i], At, g["B"][i], g["C"][i], Dskip=Dk, z_t=g["z"][i], delta_bias=bias,
                      delta_softplus=True)
        oref, href = orc.step(href, s["u"][i], s["delta"][i], A, s["B"][i], s["C"][i], Dskip=s["Dskip"], z_t=s["z"][i],
                              bias=s["delta_bias"], softplus=True)
        util.assert_close(o, oref, "bf16", "out_t")
    util.assert_close(h, href, "bf16", "h")


def test_layer_with_32_states():
    import torch
    from paper_2312_00752_amd import binding as B
    w = wl.make_layer_inputs(2, 200, 96, 32, "bf16", seed=35, rank=4)
    rng = np.random.default_rng(36)
    w["A"] = -np.exp(rng.uniform(np.log(0.02), np.log(8.0), size=(96, 32))).astype(np.float32)
    names = ("x", "z", "conv_w", "conv_b", "W_x", "W_dt", "dt_bias", "A", "Dskip")
    t = {k: torch.from_numpy(w[k]).cuda() for k in names + ("dout",)}
    for k in ("x", "z", "W_x", "W_dt", "dout"):
        t[k] = t[k].to(torch.bfloat16)
    saved = torch.empty(B.ss_layer_saved_bytes(2, 96, 200, 32, 4), dtype=torch.uint8, device="cuda")
    scratch = torch.empty(B.ss_layer_scratch_bytes(2, 96, 200, 32, 4), dtype=torch.uint8, device="cuda")
    args = [t[k] for k in names]
    out = B.ss_layer_fwd(*args, scratch=scratch, saved=saved)
    out_plain = B.ss_layer_fwd(*args, scratch=scratch)
    g = B.ss_layer_bwd(t["dout"], *args, scratch=scratch, saved=saved)
    torch.cuda.synchronize()
    rnd = lambda a: wl.round_to_bf16(a).astype(np.float64)
    kw = {k: w[k] for k in names}
    ref = inn.inner_fwd(rnd=rnd, **kw)
    rg = inn.inner_bwd(dout=w["dout"], rnd=rnd, **kw)
    util.assert_close(out, ref["out"], "bf16", "out", exact_inputs=False)
    util.assert_close(out_plain, ref["out"], "bf16", "out (nothing saved)", exact_inputs=False)
    for k in ("dx", "dz", "dconv_w", "dconv_b", "dW_x", "dW_dt", "ddt_bias", "dA", "dD"):
        util.assert_close(g[k], rg[k], "bf16", k, exact_inputs=False)
