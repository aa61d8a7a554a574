"""Complex-valued state on the GPU (SS_COMPLEX_STATE; Section 3.6 "Real vs. Complex", S4D-Lin
initialisation A_n = -1/2 + n i) against the complex128 oracle: forward, backward, step, split
sequences, more than 8 complex states, time-invariant B / C."""
import numpy as np
import pytest

from oracle import complex_oracle as cx
from paper_2312_00752_amd import workloads as wl
from tests import util

pytestmark = pytest.mark.gpu


def _pairs_last(a):
    """complex (..., n) -> float32 (..., n, 2)"""
    return np.ascontiguousarray(np.stack([np.real(a), np.imag(a)], axis=-1), dtype=np.float32)


def _pairs_before_time(a):
    """complex (B, N, L) -> float32 (B, N, 2, L)"""
    return np.ascontiguousarray(np.stack([np.real(a), np.imag(a)], axis=2), dtype=np.float32)


def _workload(io, batch, seqlen, dim, dstate, seed, s4d_lin):
    rng = np.random.default_rng(seed)
    rnd = (lambda a: wl.round_to_bf16(a)) if io == "bf16" else (lambda a: a.astype(np.float32))
    n = lambda *s: rng.standard_normal(s).astype(np.float32)
    w = {"io": io, "u": rnd(n(batch, dim, seqlen)), "delta": rnd(n(batch, dim, seqlen)), "z": rnd(n(batch, dim, seqlen)),
         "dout": rnd(n(batch, dim, seqlen))}
    if s4d_lin:
        A = np.broadcast_to(-0.5 + 1j * np.arange(dstate), (dim, dstate)).astype(np.complex64)
    else:
        A = (-np.exp(rng.uniform(np.log(0.05), np.log(4.0), size=(dim, dstate))) + 1j * rng.normal(size=(dim, dstate)) * 3.0).astype(np.complex64)
    w["A"] = A
    scale = np.float32(1.0 / np.sqrt(max(dstate / 8.0, 1.0)))
    w["B"] = rnd(n(batch, dstate, seqlen)) + 1j * rnd(n(batch, dstate, seqlen))
    w["C"] = rnd(n(batch, dstate, seqlen) * scale) + 1j * rnd(n(batch, dstate, seqlen) * scale)
    w["Dskip"] = n(dim)
    w["delta_bias"] = np.log(np.expm1(rng.uniform(1e-3, 1e-1, size=dim))).astype(np.float32)
    w["h0"] = (n(batch, dim, dstate) + 1j * n(batch, dim, dstate)).astype(np.complex64)
    w["dh_last"] = (n(batch, dim, dstate) + 1j * n(batch, dim, dstate)).astype(np.complex64)
    return w


def _upload(w):
    import torch
    io = torch.bfloat16 if w["io"] == "bf16" else torch.float32
    g = {k: torch.from_numpy(w[k]).cuda().to(io) for k in ("u", "delta", "z", "dout")}
    g["A"] = torch.from_numpy(_pairs_last(w["A"])).cuda()
    g["h0"] = torch.from_numpy(_pairs_last(w["h0"])).cuda()
    g["dh_last"] = torch.from_numpy(_pairs_last(w["dh_last"])).cuda()
    for k in ("B", "C"):
        g[k] = (torch.from_numpy(_pairs_last(w[k])).cuda() if w[k].ndim == 2
                else torch.from_numpy(_pairs_before_time(w[k])).cuda().to(io))
    g["Dskip"], g["delta_bias"] = torch.from_numpy(w["Dskip"]).cuda(), torch.from_numpy(w["delta_bias"]).cuda()
    return g


def _check(w, gate=True):
    import torch
    from paper_2312_00752_amd import binding as B
    io = w["io"]
    batch, dim, seqlen = w["u"].shape
    dstate = w["A"].shape[1]
    g = _upload(w)
    code = B.SS_BF16 if io == "bf16" else B.SS_F32
    bfix, cfix = w["B"].ndim == 2, w["C"].ndim == 2
    ws = torch.empty(B.ss_workspace_bytes(batch, dim, seqlen, dstate, io_dtype=code, has_z=gate, b_fixed=bfix, c_fixed=cfix,
                                          complex_state=True), dtype=torch.uint8, device="cuda")
    kw = dict(Dskip=g["Dskip"], z=g["z"] if gate else None, delta_bias=g["delta_bias"], h0=g["h0"], delta_softplus=True,
              complex_state=True)
    out, h_last = B.ss_scan_fwd(g["u"], g["delta"], g["A"], g["B"], g["C"], return_last_state=True, workspace=ws, **kw)
    grads = B.ss_scan_bwd(g["dout"], g["u"], g["delta"], g["A"], g["B"], g["C"], ws, dh_last=g["dh_last"], want_dh0=True, **kw)
    torch.cuda.synchronize()
    okw = dict(Dskip=w["Dskip"], z=w["z"] if gate else None, bias=w["delta_bias"], h0=w["h0"], softplus=True)
    ref_f = cx.scan_fwd(w["u"], w["delta"], w["A"], w["B"], w["C"], **okw)
    ref_b = cx.scan_bwd(w["u"], w["delta"], w["A"], w["B"], w["C"], w["dout"], dh_last=w["dh_last"], **okw)
    util.assert_close(out, ref_f["out"], io, "out")
    util.assert_close(h_last, _pairs_last(ref_f["h_last"]), io, "h_last")
    for k, name in (("du", "du"), ("ddelta", "ddelta"), ("dz", "dz"), ("dD", "dD"), ("ddelta_bias", "dbias")):
        if grads[k] is not None:
            util.assert_close(grads[k], ref_b[name], io, k)
    util.assert_close(grads["dA"], _pairs_last(ref_b["dA"]), io, "dA")
    util.assert_close(grads["dh0"], _pairs_last(ref_b["dh0"]), io, "dh0")
    util.assert_close(grads["dB"], _pairs_before_time(ref_b["dB"]), io, "dB")
    util.assert_close(grads["dC"], _pairs_before_time(ref_b["dC"]), io, "dC")


@pytest.mark.parametrize("io,batch,seqlen,dim,dstate,s4d_lin,gate", [
    ("f32", 2, 160, 70, 8, True, True), ("bf16", 2, 264, 100, 8, False, True), ("f32", 1, 77, 20, 3, False, True),
    ("bf16", 3, 203, 65, 5, True, True), ("f32", 1, 4096, 64, 8, False, True), ("f32", 2, 200, 64, 16, True, False),
    ("bf16", 1, 512, 128, 32, False, True), ("f32", 2, 2100, 64, 12, False, True),
])
def test_complex_forward_and_backward(io, batch, seqlen, dim, dstate, s4d_lin, gate):
    _check(_workload(io, batch, seqlen, dim, dstate, 900 + seqlen, s4d_lin), gate)


def test_complex_time_invariant_bc():
    """S4D-style layer: complex A, B, C all parameters of shape (D,N) (Algorithm 1 over the complex numbers)."""
    import torch
    from paper_2312_00752_amd import binding as B
    w = _workload("f32", 2, 300, 66, 8, 950, True)
    rng = np.random.default_rng(951)
    Bp = (rng.normal(size=(66, 8)) + 1j * rng.normal(size=(66, 8))).astype(np.complex64)
    Cp = (rng.normal(size=(66, 8)) + 1j * rng.normal(size=(66, 8))).astype(np.complex64)
    w["B"], w["C"] = Bp, Cp
    g = _upload(w)
    ws = torch.empty(B.ss_workspace_bytes(2, 66, 300, 8, io_dtype=B.SS_F32, b_fixed=True, c_fixed=True, complex_state=True),
                     dtype=torch.uint8, device="cuda")
    kw = dict(Dskip=g["Dskip"], z=g["z"], delta_bias=g["delta_bias"], delta_softplus=True, complex_state=True)
    out, _ = B.ss_scan_fwd(g["u"], g["delta"], g["A"], g["B"], g["C"], workspace=ws, **kw)
    grads = B.ss_scan_bwd(g["dout"], g["u"], g["delta"], g["A"], g["B"], g["C"], ws, **kw)
    torch.cuda.synchronize()
    # the oracle has no time-invariant mode: run it channel by channel on broadcast copies
    for d in (0, 17, 65):
        sl = slice(d, d + 1)
        Bd = np.broadcast_to(Bp[d][None, :, None], (2, 8, 300))
        Cd = np.broadcast_to(Cp[d][None, :, None], (2, 8, 300))
        okw = dict(Dskip=w["Dskip"][sl], z=w["z"][:, sl], bias=w["delta_bias"][sl], softplus=True)
        rf = cx.scan_fwd(w["u"][:, sl], w["delta"][:, sl], w["A"][sl], Bd, Cd, **okw)
        rb = cx.scan_bwd(w["u"][:, sl], w["delta"][:, sl], w["A"][sl], Bd, Cd, w["dout"][:, sl], **okw)
        util.assert_close(out[:, sl], rf["out"], "f32", "out")
        util.assert_close(grads["du"][:, sl], rb["du"], "f32", "du")
        util.assert_close(grads["ddelta"][:, sl], rb["ddelta"], "f32", "ddelta")
        util.assert_close(grads["dA"][sl], _pairs_last(rb["dA"]), "f32", "dA")
        util.assert_close(grads["dB"][d], _pairs_last(rb["dB"].sum(axis=(0, 2))), "f32", "dB")
        util.assert_close(grads["dC"][d], _pairs_last(rb["dC"].sum(axis=(0, 2))), "f32", "dC")


@pytest.mark.parametrize("dstate", [3, 8, 20])
def test_complex_step(dstate):
    import torch
    from paper_2312_00752_amd import binding as B
    nb, nd, tokens = 3, 40, 9
    w = _workload("bf16", nb, tokens, nd, dstate, 960 + dstate, dstate == 8)
    g = _upload(w)
    h = g["h0"].clone()
    href = w["h0"]
    for t in range(tokens):
        o = B.ss_step(h, g["u"][:, :, t].contiguous(), g["delta"][:, :, t].contiguous(), g["A"],
                      g["B"][:, :, :, t].contiguous(), g["C"][:, :, :, t].contiguous(), Dskip=g["Dskip"],
                      z_t=g["z"][:, :, t].contiguous(), delta_bias=g["delta_bias"], delta_softplus=True, complex_state=True)
        oref, href = cx.step(href, w["u"][:, :, t], w["delta"][:, :, t], w["A"], w["B"][:, :, t], w["C"][:, :, t],
                             Dskip=w["Dskip"], z_t=w["z"][:, :, t], bias=w["delta_bias"], softplus=True)
        util.assert_close(o, oref, "bf16", "out_t")
    util.assert_close(h, _pairs_last(href), "bf16", "h")


def test_complex_with_exact_zoh_is_refused():
    import torch
    from paper_2312_00752_amd import binding as B
    w = _workload("f32", 1, 16, 8, 2, 970, True)
    g = _upload(w)
    with pytest.raises(B.SsError):
        B.ss_scan_fwd(g["u"], g["delta"], g["A"], g["B"], g["C"], complex_state=True, exact_zoh=True)
