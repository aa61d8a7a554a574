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
    errs, elem = {}, {}
    ref = util.oracle_fwd(w)
    for k, got in (("out", out), ("h_last", h_last)):
        errs[k] = util.assert_close(got, ref[k], io, k)
        elem[k] = util.elem_err(got, ref[k])
    del ref, out, h_last
    gc.collect()
    ref = util.oracle_bwd(w)
    for k in GRADS:
        errs[k] = util.assert_close(grads[k], ref[ORACLE_NAME.get(k, k)], io, k)
        elem[k] = util.elem_err(grads[k], ref[ORACLE_NAME.get(k, k)])
        grads[k] = None
    print(name, "max|diff|/max|ref|:", {k: "%.1e" % v for k, v in errs.items()})
    print(name, "max_i |diff_i| / (|ref_i| + %.2f max|ref|):" % util.ELEM_FLOOR, {k: "%.1e" % v for k, v in elem.items()})


def test_full_size_decode_steps():
    """4096 single-token steps at batch 64, D 4096, N 16 (bf16 I/O) through ss_step, checked
    against the oracle's scan on a sample of channels (rows are independent, so the
    oracle can compute any subset of them on its own)."""
    import torch
    from oracle import ss_oracle as orc
    from paper_2312_00752_amd import binding as B
    nb, nd, nn, tokens, seed = wl.STEP_CONFIG[0], wl.STEP_CONFIG[1], wl.STEP_CONFIG[2], wl.STEP_CONFIG[4], wl.STEP_CONFIG[5]
    rng = np.random.default_rng(seed)
    sample = np.sort(rng.choice(nd, size=48, replace=False))
    f32, bf = torch.float32, torch.bfloat16
    A = -np.broadcast_to(np.arange(1, nn + 1, dtype=np.float32), (nd, nn)).copy()
    Dskip = rng.standard_normal(nd, dtype=np.float32)
    bias = np.log(np.expm1(rng.uniform(1e-3, 1e-1, size=nd))).astype(np.float32)
    gA, gD, gb = (torch.from_numpy(a).cuda() for a in (A, Dskip, bias))
    h = torch.zeros(nb, nd, nn, device="cuda", dtype=f32)
    keep = {k: [] for k in ("u", "delta", "z", "B", "C", "out")}
    chunk = 128
    for c0 in range(0, tokens, chunk):
        # the recipe of make_step_inputs, drawn chunk by chunk to bound host memory
        s = {k: wl.round_to_bf16(rng.standard_normal((chunk, nb, nd), dtype=np.float32)) for k in ("u", "z", "delta")}
        s.update({k: wl.round_to_bf16(rng.standard_normal((chunk, nb, nn), dtype=np.float32)) for k in ("B", "C")})
        g = {k: torch.from_numpy(v).cuda().to(bf) for k, v in s.items()}
        outs = []
        for t in range(chunk):
            outs.append(B.ss_step(h, g["u"][t], g["delta"][t], gA, g["B"][t], g["C"][t], Dskip=gD,
                                  z_t=g["z"][t], delta_bias=gb, delta_softplus=True))
        torch.cuda.synchronize()
        for k in ("u", "delta", "z"):
            keep[k].append(s[k][:, :, sample])
        for k in ("B", "C"):
            keep[k].append(s[k])
        keep["out"].append(torch.stack(outs)[:, :, sample].float().cpu().numpy())
    cat = lambda k: np.concatenate(keep[k], axis=0)
    tbd = lambda a: np.ascontiguousarray(a.transpose(1, 2, 0))          # (T,B,X) -> (B,X,T)
    ref = orc.scan_fwd(tbd(cat("u")), tbd(cat("delta")), A[sample], tbd(cat("B")), tbd(cat("C")),
                       Dskip=Dskip[sample], z=tbd(cat("z")), bias=bias[sample], softplus=True)
    util.assert_close(tbd(cat("out")), ref["out"], "bf16", "step outputs")
    util.assert_close(h[:, sample], ref["h_last"], "f32", "final state")
