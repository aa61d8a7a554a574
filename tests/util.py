"""Helpers shared by the GPU parity tests: upload a workload, run the oracle, compare."""
import numpy as np

from oracle import ss_oracle as orc

# Tolerances of the benchmark spec, per output tensor: max |gpu - oracle| / max |oracle| at most
# 1e-4 for float32 I/O and 2e-2 for bf16 I/O (float32 state).  A tensor the library produces in
# float32 (h_last, dB, dC, dA, dD, ddelta_bias, dh0) is held to 1e-4 in a bf16 workload too: the
# bf16 inputs are exact for the oracle, and state and sums are float32 on both sides.
TOL = {"f32": 1e-4, "bf16": 2e-2}
# Element-wise criterion beside it: |gpu - oracle| <= tol * (|oracle| + ELEM_FLOOR * max |oracle|)
# for every element, so that elements far below the tensor's peak are checked against their own
# size down to a floor (sums of terms of the peak's size cancel to small values whose float32
# error is relative to the terms; the floor leaves room for that).  Where io-dtype roundings lie
# inside the operation (the layer's intermediates; the pre-gate output accumulated over the passes
# of more than 16 states) small results carry bf16-sized errors of the terms: floor ELEM_FLOOR_ROUNDED.
ELEM_FLOOR = 0.05
ELEM_FLOOR_ROUNDED = 0.25


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


def _as_f64(got):
    return got.detach().float().cpu().numpy().astype(np.float64) if hasattr(got, "detach") else np.asarray(got, np.float64)


def rel_err(got, ref):
    """Scale-relative error of a tensor: max |got - ref| / max |ref|."""
    got = _as_f64(got)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    scale = np.max(np.abs(ref))
    err = np.max(np.abs(got - ref))
    if not np.isfinite(err):
        return float("inf")
    return float(err / scale) if scale > 0 else float(err)


def elem_err(got, ref, floor=ELEM_FLOOR):
    """Worst element-wise error: max_i |got_i - ref_i| / (|ref_i| + floor * max |ref|)."""
    got = _as_f64(got)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    scale = np.max(np.abs(ref))
    if scale == 0:
        return float(np.max(np.abs(got)))
    ratio = np.abs(got - ref) / (np.abs(ref) + floor * scale)
    worst = np.max(ratio)
    return float(worst) if np.isfinite(worst) else float("inf")


def tolerance(got, io, exact_inputs=True):
    """The limit a produced tensor is held to (see TOL).  ``exact_inputs=False``: the operation
    rounds intermediates to the io dtype between its kernels (the layer), so its float32 results
    carry bf16-sized differences wherever the two sides round a value to different neighbours."""
    import torch
    if io == "bf16" and exact_inputs and hasattr(got, "dtype") and got.dtype == torch.float32:
        return TOL["f32"]
    return TOL[io]


def assert_close(got, ref, io, name, exact_inputs=True, elem_floor=None):
    """Both criteria (see TOL, ELEM_FLOOR); returns the scale-relative error."""
    tol = tolerance(got, io, exact_inputs)
    floor = elem_floor if elem_floor is not None else (ELEM_FLOOR if exact_inputs else ELEM_FLOOR_ROUNDED)
    e = rel_err(got, ref)
    assert e <= tol, "%s: scale-relative error %.3e exceeds %.1e" % (name, e, tol)
    ee = elem_err(got, ref, floor)
    assert ee <= tol, "%s: element-wise error %.3e (of |ref| + %.2f max|ref|) exceeds %.1e" % (name, ee, floor, tol)
    return e
