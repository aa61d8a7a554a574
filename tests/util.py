"""Helpers shared by the GPU parity tests: upload a workload, run the oracle, compare."""
import numpy as np

from oracle import ss_oracle as orc

TOL = {"f32": 1e-4, "bf16": 2e-2}   # max |gpu - oracle| / max |oracle| per tensor


def upload(w, device="cuda"):
    """Workload dict of float32 numpy arrays -> dict of CUDA tensors in the io dtype."""
    import torch
    io = torch.bfloat16 if w["io"] == "bf16" else torch.float32
    g = {}
    for k in ("u", "delta", "z", "B", "C", "dout"):
        g[k] = None if w.get(k) is None else torch.from_numpy(w[k]).to(device).to(io).contiguous()
    for k in ("A", "Dskip", "delta_bias", "h0", "dh_last"):
        g[k] = None if w.get(k) is None else torch.from_numpy(np.asarray(w[k], dtype=np.float32)).to(device).contiguous()
    return g


def oracle_fwd(w, nthreads=0):
    return orc.scan_fwd(w["u"], w["delta"], w["A"], w["B"], w["C"], Dskip=w.get("Dskip"),
                        z=w.get("z"), bias=w.get("delta_bias"), h0=w.get("h0"),
                        softplus=w.get("delta_softplus", False), nthreads=nthreads)


def oracle_bwd(w, nthreads=0):
    return orc.scan_bwd(w["u"], w["delta"], w["A"], w["B"], w["C"], w["dout"], Dskip=w.get("Dskip"),
                        z=w.get("z"), bias=w.get("delta_bias"), h0=w.get("h0"),
                        dh_last=w.get("dh_last"), softplus=w.get("delta_softplus", False),
                        nthreads=nthreads)


def rel_err(got, ref):
    """Scale-relative error of a tensor: max |got - ref| / max |ref|."""
    got = got.detach().float().cpu().numpy().astype(np.float64) if hasattr(got, "detach") else np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    scale = np.max(np.abs(ref))
    err = np.max(np.abs(got - ref))
    if not np.isfinite(err):
        return float("inf")
    return float(err / scale) if scale > 0 else float(err)


def assert_close(got, ref, io, name):
    e = rel_err(got, ref)
    assert e <= TOL[io], "%s: scale-relative error %.3e exceeds %.1e" % (name, e, TOL[io])
    return e
