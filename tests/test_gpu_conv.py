"""GPU parity of the short causal convolution (+ SiLU) against the float64 oracle."""
import numpy as np
import pytest

from oracle import conv_oracle as cv
from paper_2312_00752_amd.workloads import make_conv_inputs
from tests.util import assert_close

pytestmark = pytest.mark.gpu


def _up(a, io):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.to(torch.bfloat16) if io == "bf16" else t


def _run(w, silu=True, with_bias=True, with_state=False):
    from paper_2312_00752_amd import binding as B
    io = w["io"]
    x, wt = _up(w["x"], io), _up(w["w"], "f32")
    bias = _up(w["bias"], "f32") if with_bias else None
    st = _up(w["state_in"], io) if with_state else None
    out, state_out = B.ss_conv_fwd(x, wt, bias, st, silu=silu, return_state=True)
    g = B.ss_conv_bwd(_up(w["dout"], io), x, wt, bias, st, silu=silu)
    return out, state_out, g


def _check(w, silu=True, with_bias=True, with_state=False):
    out, state_out, g = _run(w, silu, with_bias, with_state)
    bias = w["bias"] if with_bias else None
    st = w["state_in"] if with_state else None
    ref = cv.conv_fwd(w["x"], w["w"], bias, st, silu)
    rg = cv.conv_bwd(w["x"], w["w"], w["dout"], bias, st, silu)
    tol = w["io"]
    assert_close(out, ref["out"], tol, "out")
    if w["shape"][3] > 1:
        # the window is a copy of inputs: exact
        np.testing.assert_array_equal(state_out.float().cpu().numpy(), ref["state_out"].astype(np.float32))
    assert_close(g["dx"], rg["dx"], tol, "dx")
    assert_close(g["dw"], rg["dw"], tol, "dw")
    if with_bias:
        assert_close(g["dbias"], rg["dbias"], tol, "dbias")


@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("L", [1, 2, 3, 7, 8, 13, 64, 511, 512, 513, 520, 1000, 1032, 2056])
def test_conv_lengths(io, L):
    _check(make_conv_inputs(2, 5, L, 4, io, seed=L), with_state=(L % 2 == 1))


@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("W", [1, 2, 3, 4])
@pytest.mark.parametrize("silu,with_bias,with_state", [(True, True, True), (False, False, False),
                                                      (True, False, True), (False, True, False)])
def test_conv_widths_and_flags(io, W, silu, with_bias, with_state):
    _check(make_conv_inputs(3, 70, 776, W, io, seed=10 * W), silu, with_bias, with_state)
    _check(make_conv_inputs(1, 3, 21, W, io, seed=10 * W + 1), silu, with_bias, with_state)


def test_conv_many_channels_few_steps_and_few_channels_many_steps():
    _check(make_conv_inputs(2, 3000, 40, 4, "bf16", seed=3))
    _check(make_conv_inputs(1, 2, 300000, 4, "f32", seed=4), with_state=True)


@pytest.mark.parametrize("io", ["f32", "bf16"])
def test_conv_in_pieces_and_token_by_token(io):
    import torch
    from paper_2312_00752_amd import binding as B
    w = make_conv_inputs(2, 96, 1064, 4, io, seed=7)
    x, wt, bias = _up(w["x"], io), _up(w["w"], "f32"), _up(w["bias"], "f32")
    whole, st_whole = B.ss_conv_fwd(x, wt, bias, return_state=True)
    cut = 1000
    a, st = B.ss_conv_fwd(x[:, :, :cut].contiguous(), wt, bias, return_state=True)
    b, st2 = B.ss_conv_fwd(x[:, :, cut:].contiguous(), wt, bias, state_in=st, return_state=True)
    assert torch.equal(torch.cat([a, b], 2), whole)
    assert torch.equal(st2, st_whole)
    # decode: continue token by token from the state after `cut` steps
    state = st.clone()
    for t in range(cut, 1064):
        o = B.ss_conv_step(state, x[:, :, t].contiguous(), wt, bias)
        assert torch.equal(o, whole[:, :, t]), t
    assert torch.equal(state, st_whole)
    ref = cv.conv_fwd(w["x"], w["w"], w["bias"])
    assert_close(whole, ref["out"], io, "out")


@pytest.mark.parametrize("W", [2, 3])
def test_conv_step_narrow_widths(W):
    import torch
    from paper_2312_00752_amd import binding as B
    w = make_conv_inputs(2, 33, 19, W, "f32", seed=W)
    x, wt = _up(w["x"], "f32"), _up(w["w"], "f32")
    state = torch.zeros(2, 33, W - 1, device="cuda")
    ref = cv.conv_fwd(w["x"], w["w"], None, None, silu=False)
    for t in range(19):
        o = B.ss_conv_step(state, x[:, :, t].contiguous(), wt, None, silu=False)
        assert_close(o, ref["out"][:, :, t], "f32", "out_t")
    np.testing.assert_array_equal(state.cpu().numpy(), ref["state_out"].astype(np.float32))


def test_conv_empty_sequence():
    import torch
    from paper_2312_00752_amd import binding as B
    wt = torch.randn(8, 4, device="cuda")
    x = torch.empty(2, 8, 0, device="cuda", dtype=torch.bfloat16)
    st = torch.randn(2, 8, 3, device="cuda").to(torch.bfloat16)
    out, so = B.ss_conv_fwd(x, wt, None, state_in=st, return_state=True)
    assert out.shape == (2, 8, 0) and torch.equal(so, st)
    out, so = B.ss_conv_fwd(x, wt, None, return_state=True)
    assert torch.count_nonzero(so) == 0
    g = B.ss_conv_bwd(x, x, wt, None)
    assert torch.count_nonzero(g["dw"]) == 0


def test_conv_full_size_layer_shape():
    """The headline layer shape (8, 4096, 2048) in bf16, compared element by element."""
    _check(make_conv_inputs(8, 4096, 2048, 4, "bf16", seed=2))
