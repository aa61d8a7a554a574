"""Randomised parity sweep: shapes, dtypes and optional inputs drawn from a fixed seed."""
import numpy as np
import pytest

from paper_2312_00752_amd import workloads as wl
from tests import util
from tests.test_gpu_bwd import GRADS, ORACLE_NAME

pytestmark = pytest.mark.gpu


def _cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        long_seq = i % 4 == 3            # every fourth case is long enough to be split
        out.append(dict(
            batch=int(rng.integers(1, 4)), dim=int(rng.integers(1, 40 if long_seq else 200)),
            seqlen=int(rng.integers(2048, 3300)) if long_seq else int(rng.integers(1, 700)),
            dstate=int(rng.integers(1, 17)), io=str(rng.choice(["f32", "bf16"])),
            with_z=bool(rng.integers(0, 2)), with_D=bool(rng.integers(0, 2)), with_bias=bool(rng.integers(0, 2)),
            softplus=bool(rng.integers(0, 4) > 0), h0=bool(rng.integers(0, 2)), dh_last=bool(rng.integers(0, 2)),
            align8=bool(rng.integers(0, 2)), seed=1000 + i))
    return out


@pytest.mark.parametrize("case", _cases(24, 7), ids=lambda c: "b%(batch)d_d%(dim)d_l%(seqlen)d_n%(dstate)d_%(io)s" % c)
def test_random_case(case):
    import torch
    from paper_2312_00752_amd import binding as B
    nb, nd, nn, io = case["batch"], case["dim"], case["dstate"], case["io"]
    nl = case["seqlen"] // 8 * 8 if case["align8"] and case["seqlen"] >= 8 else case["seqlen"]
    w = wl.make_scan_inputs(nb, nl, nd, nn, io=io, seed=case["seed"], with_z=case["with_z"],
                            with_D=case["with_D"], with_bias=case["with_bias"])
    rng = np.random.default_rng(case["seed"] + 1)
    if not case["softplus"]:
        w["delta_softplus"] = False
        w["delta"] = np.abs(w["delta"]) * np.float32(0.1)
        if io == "bf16":
            w["delta"] = wl.round_to_bf16(w["delta"])
        if w["delta_bias"] is not None:
            w["delta_bias"] = np.abs(w["delta_bias"]) * np.float32(0.01)
    # a non-trivial A (negative, not the initialisation pattern)
    w["A"] = (-np.exp(rng.normal(size=(nd, nn)))).astype(np.float32)
    if case["h0"]:
        w["h0"] = rng.normal(size=(nb, nd, nn)).astype(np.float32)
    if case["dh_last"]:
        w["dh_last"] = rng.normal(size=(nb, nd, nn)).astype(np.float32)
    g = util.upload(w)
    code = B.SS_BF16 if io == "bf16" else B.SS_F32
    ws = torch.empty(max(256, B.ss_workspace_bytes(nb, nd, nl, nn, io_dtype=code)), dtype=torch.uint8, device="cuda")
    kw = dict(Dskip=g["Dskip"], z=g["z"], delta_bias=g["delta_bias"], h0=g["h0"],
              delta_softplus=w["delta_softplus"])
    out, h_last = B.ss_scan_fwd(g["u"], g["delta"], g["A"], g["B"], g["C"], return_last_state=True,
                                workspace=ws, **kw)
    grads = B.ss_scan_bwd(g["dout"], g["u"], g["delta"], g["A"], g["B"], g["C"], ws,
                          dh_last=g["dh_last"], want_dh0=True, **kw)
    torch.cuda.synchronize()
    ref_f, ref_b = util.oracle_fwd(w), util.oracle_bwd(w)
    util.assert_close(out, ref_f["out"], io, "out")
    util.assert_close(h_last, ref_f["h_last"], io, "h_last")
    for k in GRADS:
        r = ref_b[ORACLE_NAME.get(k, k)]
        if r is None:
            assert grads[k] is None
        else:
            util.assert_close(grads[k], r, io, k)
