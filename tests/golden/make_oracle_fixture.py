"""Writes tests/golden/oracle_tiny_case.npz-like text fixture from the oracle alone.

Run from the repository root:  python tests/golden/make_oracle_fixture.py
The stored numbers guard the oracle's arithmetic against accidental change (they are the
oracle's own output, so they pin nothing by themselves; the closed-form pins do that)."""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import ss_oracle as orc  # noqa: E402
from paper_2312_00752_amd import workloads as wl  # noqa: E402


def case():
    w = wl.make_scan_inputs(2, 12, 3, 4, io="f32", seed=123)
    rng = np.random.default_rng(124)
    w["A"] = (-np.exp(rng.normal(size=(3, 4)))).astype(np.float32)
    return w


def compute(w, exact_zoh):
    kw = dict(Dskip=w["Dskip"], z=w["z"], bias=w["delta_bias"], softplus=True, exact_zoh=exact_zoh)
    f = orc.scan_fwd(w["u"], w["delta"], w["A"], w["B"], w["C"], **kw)
    b = orc.scan_bwd(w["u"], w["delta"], w["A"], w["B"], w["C"], w["dout"], **kw)
    return {"out": f["out"], "h_last": f["h_last"], "du": b["du"], "ddelta": b["ddelta"], "dz": b["dz"],
            "dB": b["dB"], "dC": b["dC"], "dA": b["dA"], "dD": b["dD"], "dbias": b["dbias"]}


if __name__ == "__main__":
    w = case()
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_tiny_case.txt")
    with open(path, "w") as fh:
        fh.write("# oracle output on workloads.make_scan_inputs(2, 12, 3, 4, 'f32', seed=123) with A = -exp(N(0,1)), seed 124\n")
        fh.write("# written by tests/golden/make_oracle_fixture.py (calls only oracle/); one tensor per line: name mode values...\n")
        for zoh in (False, True):
            for name, arr in compute(w, zoh).items():
                fh.write("%s %s %s\n" % (name, "zoh" if zoh else "first_order",
                                         " ".join("%.17g" % v for v in np.asarray(arr).reshape(-1))))
    print("wrote", path)
