"""GPU parity of ss_scan_fwd and ss_step against the float64 oracle (needs an MI355X)."""
import numpy as np
import pytest

from paper_2312_00752_amd import workloads as wl
from tests import util

pytestmark = pytest.mark.gpu


def _gpu_fwd(w, g=None, **kw):
    from paper_2312_00752_amd import binding as B
    import torch
    g = g or util.upload(w)
    out, h_last = B.ss_scan_fwd(g["u"], g["delta"], g["A"], g["B"], g["C"], Dskip=g["Dskip"], z=g["z"],
                                delta_bias=g["delta_bias"], h0=g["h0"],
                                delta_softplus=w.get("delta_softplus", False),
                                return_last_state=True, **kw)
    torch.cuda.synchronize()
    return out, h_last


def _check_fwd(w):
    out, h_last = _gpu_fwd(w)
    ref = util.oracle_fwd(w)
    e1 = util.assert_close(out, ref["out"], w["io"], "out")
    e2 = util.assert_close(h_last, ref["h_last"], "f32" if w["io"] == "f32" else "bf16", "h_last")
    return e1, e2


def test_config0_tiny_fp32_full():
    _check_fwd(wl.make_config("tiny_fp32"))


@pytest.mark.parametrize("name,batch,seqlen,dim", [
    ("mamba130m_layer_bf16", 2, 2048, 192),     # whole chunks, 3 row tiles
    ("mamba1p4b_layer_bf16", 2, 264, 100),      # ragged row tile; 8-aligned tail chunk
    ("mamba2p8b_long_bf16", 1, 4104, 70),       # many chunks, log-uniform step sizes
    ("genomics_1m_fp32", 1, 8192, 256),         # fp32 I/O, one-hot-like input
    ("mamba1p4b_layer_bf16", 3, 203, 65),       # nothing aligned: element-wise path
    ("tiny_fp32", 2, 77, 5),                    # fp32 element-wise path
])
def test_scaled_configs(name, batch, seqlen, dim):
    _check_fwd(wl.make_config(name, scale_batch=batch, scale_seqlen=seqlen, scale_dim=dim))


@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("dstate", [1, 3, 4, 8, 13, 16])
def test_state_sizes(io, dstate):
    _check_fwd(wl.make_scan_inputs(2, 96, 70, dstate, io=io, seed=30 + dstate))


@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("drop", ["z", "Dskip", "delta_bias", "softplus", "all"])
def test_optional_inputs(io, drop):
    w = wl.make_scan_inputs(2, 160, 33, 16, io=io, seed=40)
    if drop in ("z", "all"):
        w["z"] = None
    if drop in ("Dskip", "all"):
        w["Dskip"] = None
    if drop in ("delta_bias", "all"):
        w["delta_bias"] = None
    if drop in ("softplus", "all"):
        w["delta_softplus"] = False
        w["delta"] = np.abs(w["delta"]) * np.float32(0.1)   # used as the step size directly
        if io == "bf16":
            w["delta"] = wl.round_to_bf16(w["delta"])
        if w["delta_bias"] is not None:
            w["delta_bias"] = np.abs(w["delta_bias"]) * np.float32(0.01)
    _check_fwd(w)


@pytest.mark.parametrize("seqlen", [1, 2, 7, 8, 31, 32, 33, 64])
def test_short_sequences(seqlen):
    _check_fwd(wl.make_scan_inputs(2, seqlen, 20, 16, io="f32", seed=50 + seqlen))


def test_empty_sequence_returns_initial_state():
    import torch
    from paper_2312_00752_amd import binding as B
    w = wl.make_scan_inputs(2, 8, 6, 16, io="f32", seed=60)
    g = util.upload(w)
    h0 = torch.randn(2, 6, 16, device="cuda")
    empty = lambda t: t[..., :0].contiguous()
    out, h_last = B.ss_scan_fwd(empty(g["u"]), empty(g["delta"]), g["A"], empty(g["B"]), empty(g["C"]),
                                h0=h0, return_last_state=True)
    torch.cuda.synchronize()
    assert out.numel() == 0 and torch.equal(h_last, h0)
    out, h_last = B.ss_scan_fwd(empty(g["u"]), empty(g["delta"]), g["A"], empty(g["B"]), empty(g["C"]),
                                return_last_state=True)
    torch.cuda.synchronize()
    assert torch.count_nonzero(h_last) == 0


def test_initial_state_and_chunk_continuation():
    """scan(0:L) == scan(0:L1) continued from its last state (Appendix D), on the GPU."""
    import torch
    w = wl.make_scan_inputs(2, 200, 40, 16, io="f32", seed=61)
    w["h0"] = np.random.default_rng(62).normal(size=(2, 40, 16)).astype(np.float32)
    out, h_last = _gpu_fwd(w)
    ref = util.oracle_fwd(w)
    util.assert_close(out, ref["out"], "f32", "out")
    util.assert_close(h_last, ref["h_last"], "f32", "h_last")
    cut = 72
    a = {k: (v[..., :cut].copy() if k in ("u", "delta", "z", "B", "C") else v) for k, v in w.items()}
    b = {k: (v[..., cut:].copy() if k in ("u", "delta", "z", "B", "C") else v) for k, v in w.items()}
    out_a, h_a = _gpu_fwd(a)
    b["h0"] = h_a.cpu().numpy()
    out_b, h_b = _gpu_fwd(b)
    util.assert_close(torch.cat([out_a, out_b], -1), ref["out"], "f32", "out (two pieces)")
    util.assert_close(h_b, ref["h_last"], "f32", "h_last (two pieces)")


def test_forward_is_bitwise_reproducible_and_leaves_inputs_alone():
    import torch
    w = wl.make_config("mamba1p4b_layer_bf16", scale_batch=2, scale_seqlen=512, scale_dim=128)
    g = util.upload(w)
    keep = {k: v.clone() for k, v in g.items() if v is not None}
    o1, h1 = _gpu_fwd(w, g)
    o2, h2 = _gpu_fwd(w, g)
    assert torch.equal(o1, o2) and torch.equal(h1, h2)
    for k, v in keep.items():
        assert torch.equal(v, g[k]), k


@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("dstate,seqlen", [(1, 70), (13, 96), (16, 200), (16, 37), (40, 64)])
def test_repacked_operands_give_the_same_bits(io, dstate, seqlen):
    """With a workspace the forward kernels read B and C from a repacked copy, without one in
    place: same values, same order of operations, so the results must be bit-identical (the shapes
    have enough rows that the sequence is not split, which would reorder the sums)."""
    import torch
    from paper_2312_00752_amd import binding as B
    w = wl.make_scan_inputs(8, seqlen, 4096, dstate, io=io, seed=170 + dstate)
    g = util.upload(w)
    code = B.SS_BF16 if io == "bf16" else B.SS_F32
    # (more than 16 states with a gate need the workspace anyway: compare its two uses only)
    plain, h_plain = _gpu_fwd(w, g) if dstate <= 16 else (None, None)
    nbytes = B.ss_workspace_bytes(8, 4096, seqlen, dstate, for_backward=False, io_dtype=code)
    assert nbytes > 0
    ws = torch.full((nbytes,), 0xff, dtype=torch.uint8, device="cuda")       # NaN-poisoned scratch
    lent, h_lent = _gpu_fwd(w, g, workspace=ws, save_for_bwd=False)
    if plain is None:
        plain, h_plain = lent, h_lent
    assert torch.equal(plain, lent) and torch.equal(h_plain, h_lent)
    ws2 = torch.full((B.ss_workspace_bytes(8, 4096, seqlen, dstate, io_dtype=code),), 0xff, dtype=torch.uint8, device="cuda")
    saved, h_saved = _gpu_fwd(w, g, workspace=ws2, save_for_bwd=True)
    assert torch.equal(plain, saved) and torch.equal(h_plain, h_saved)


@pytest.mark.parametrize("io", ["f32", "bf16"])
def test_step_by_step_equals_scan(io):
    """L calls of ss_step from h0 reproduce ss_scan_fwd (recurrent == parallel mode, Section 2)."""
    import torch
    from paper_2312_00752_amd import binding as B
    L = 48
    w = wl.make_scan_inputs(3, L, 37, 16, io=io, seed=63)
    w["h0"] = np.random.default_rng(64).normal(size=(3, 37, 16)).astype(np.float32)
    g = util.upload(w)
    ref = util.oracle_fwd(w)
    h = g["h0"].clone()
    outs = []
    for t in range(L):
        o = B.ss_step(h, g["u"][..., t].contiguous(), g["delta"][..., t].contiguous(), g["A"],
                      g["B"][..., t].contiguous(), g["C"][..., t].contiguous(), Dskip=g["Dskip"],
                      z_t=g["z"][..., t].contiguous(), delta_bias=g["delta_bias"], delta_softplus=True)
        outs.append(o)
    torch.cuda.synchronize()
    util.assert_close(torch.stack(outs, -1), ref["out"], io, "step outputs")
    util.assert_close(h, ref["h_last"], io, "step state")
    out, h_last = _gpu_fwd(w, g)
    util.assert_close(h, h_last.cpu().numpy(), io, "step vs scan state")


# From 2 x 256 x 2048 lanes on, ss_step takes 2 or 4 batch entries of a channel per thread (N = 16): both
# counts, both dtypes, a last workgroup that is partly filled, and every optional operand absent once.
@pytest.mark.parametrize("io,batch,dim,full", [("bf16", 132, 4000, True), ("f32", 66, 4000, True), ("bf16", 68, 3900, False)])
def test_step_several_batch_entries_per_thread(io, batch, dim, full):
    import torch
    from oracle import ss_oracle as orc
    from paper_2312_00752_amd import binding as B
    s = wl.make_step_inputs(batch, dim, 16, 2, io=io, seed=71)
    h_ref = np.random.default_rng(72).normal(size=(batch, dim, 16)).astype(np.float32)
    h = torch.from_numpy(h_ref).cuda()
    h_ref = h_ref.astype(np.float64)
    tio = torch.bfloat16 if io == "bf16" else torch.float32
    up = lambda a, dt: torch.from_numpy(a).cuda().to(dt)
    for t in range(2):
        dl = s["delta"][t] if full else np.abs(s["delta"][t])   # without softplus the step size itself: keep it non-negative
        kw = dict(Dskip=up(s["Dskip"], torch.float32), z_t=up(s["z"][t], tio), delta_bias=up(s["delta_bias"], torch.float32)) if full else {}
        o = B.ss_step(h, up(s["u"][t], tio), up(dl, tio), up(s["A"], torch.float32), up(s["B"][t], tio),
                      up(s["C"][t], tio), delta_softplus=full, **kw)
        rkw = dict(Dskip=s["Dskip"], z_t=s["z"][t], bias=s["delta_bias"]) if full else {}
        o_ref, h_ref = orc.step(h_ref, s["u"][t], dl, s["A"], s["B"][t], s["C"][t], softplus=full, **rkw)
        torch.cuda.synchronize()
        util.assert_close(o, o_ref, io, "out_t")
        util.assert_close(h, h_ref, "f32", "h")


@pytest.mark.parametrize("dstate", [1, 5, 16])
def test_step_state_sizes_against_oracle(dstate):
    import torch
    from oracle import ss_oracle as orc
    from paper_2312_00752_amd import binding as B
    s = wl.make_step_inputs(5, 67, dstate, 3, io="bf16", seed=65)
    h_ref = np.random.default_rng(66).normal(size=(5, 67, dstate))
    h = torch.from_numpy(h_ref.astype(np.float32)).cuda()
    h_ref = h_ref.astype(np.float32).astype(np.float64)
    up = lambda a, dt: torch.from_numpy(a).cuda().to(dt)
    for t in range(3):
        o = B.ss_step(h, up(s["u"][t], torch.bfloat16), up(s["delta"][t], torch.bfloat16),
                      up(s["A"], torch.float32), up(s["B"][t], torch.bfloat16), up(s["C"][t], torch.bfloat16),
                      Dskip=up(s["Dskip"], torch.float32), z_t=up(s["z"][t], torch.bfloat16),
                      delta_bias=up(s["delta_bias"], torch.float32), delta_softplus=True)
        o_ref, h_ref = orc.step(h_ref, s["u"][t], s["delta"][t], s["A"], s["B"][t], s["C"][t],
                                Dskip=s["Dskip"], z_t=s["z"][t], bias=s["delta_bias"], softplus=True)
        torch.cuda.synchronize()
        util.assert_close(o, o_ref, "bf16", "out_t")
        util.assert_close(h, h_ref, "f32", "h")
