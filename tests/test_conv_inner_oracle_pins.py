"""Pins of the convolution and selective-SSM-layer oracles (CPU only).

The paper fixes the structure (Section 3.4 / Figure 3: conv -> SiLU -> SSM, gate; Algorithm
2 and Section 3.6: B, C and a low-rank Delta are linear in the conv output) but no numbers,
so the oracles are pinned to library routines on special cases (numpy.convolve, torch's
conv1d), to closed forms (impulse response, SiLU values, a layer reduced to the scan with
hand-built projections), to invariants (causality, piecewise == whole, token by token ==
whole) and to finite differences of their own pinned forward passes.
"""
import numpy as np
import pytest

from oracle import conv_oracle as cv
from oracle import inner_oracle as inn
from oracle import ss_oracle as orc


def _rng(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------- convolution --------------
@pytest.mark.parametrize("W", [2, 3, 4])
def test_conv_matches_numpy_convolve(W):
    r = _rng(W)
    x, w, b = r.normal(size=(2, 3, 19)), r.normal(size=(3, W)), r.normal(size=3)
    got = cv.conv_fwd(x, w, b, silu=False)["out"]
    for bi in range(2):
        for d in range(3):
            # cross-correlation with left padding == full convolution with the flipped taps, cut to L
            ref = np.convolve(x[bi, d], w[d, ::-1])[:19] + b[d]
            np.testing.assert_allclose(got[bi, d], ref, rtol=0, atol=1e-13)


def test_conv_matches_torch_conv1d():
    torch = pytest.importorskip("torch")
    r = _rng(11)
    x, w, b = r.normal(size=(2, 5, 33)), r.normal(size=(5, 4)), r.normal(size=5)
    ref = torch.nn.functional.conv1d(torch.from_numpy(x), torch.from_numpy(w)[:, None, :], torch.from_numpy(b),
                                     padding=3, groups=5)[..., :33]
    got = cv.conv_fwd(x, w, b, silu=True)
    np.testing.assert_allclose(got["pre"], ref.numpy(), rtol=0, atol=1e-13)
    np.testing.assert_allclose(got["out"], torch.nn.functional.silu(ref).numpy(), rtol=0, atol=1e-13)


def test_conv_impulse_response_is_the_taps_newest_last():
    w = np.array([[1.0, 2.0, 3.0, 4.0]])
    x = np.zeros((1, 1, 10))
    x[0, 0, 2] = 1.0
    out = cv.conv_fwd(x, w, silu=False)["out"][0, 0]
    # the tap with the highest index multiplies the current sample
    np.testing.assert_array_equal(out, [0, 0, 4, 3, 2, 1, 0, 0, 0, 0])


def test_silu_closed_values():
    x = np.array([[[0.0, 1.0, -1.0, 40.0, -40.0]]])
    out = cv.conv_fwd(x, np.array([[1.0]]).repeat(1, 0).reshape(1, 1), silu=True)["out"][0, 0]
    e = np.e
    np.testing.assert_allclose(out[:3], [0.0, e / (1 + e), -1 / (1 + e)], rtol=1e-15, atol=0)
    assert out[3] == pytest.approx(40.0, rel=1e-15) and abs(out[4]) < 1e-15


def test_conv_is_causal():
    r = _rng(5)
    x, w = r.normal(size=(1, 2, 16)), r.normal(size=(2, 4))
    base = cv.conv_fwd(x, w)["out"]
    x2 = x.copy()
    x2[:, :, 9] += 1.0
    out2 = cv.conv_fwd(x2, w)["out"]
    np.testing.assert_array_equal(out2[:, :, :9], base[:, :, :9])
    assert np.all(out2[:, :, 9:13] != base[:, :, 9:13])
    np.testing.assert_array_equal(out2[:, :, 13:], base[:, :, 13:])


@pytest.mark.parametrize("W,cut", [(4, 1), (4, 7), (3, 2), (2, 15)])
def test_conv_in_pieces_equals_whole(W, cut):
    r = _rng(7)
    x, w, b = r.normal(size=(2, 3, 16)), r.normal(size=(3, W)), r.normal(size=3)
    whole = cv.conv_fwd(x, w, b)
    first = cv.conv_fwd(x[:, :, :cut], w, b)
    second = cv.conv_fwd(x[:, :, cut:], w, b, state_in=first["state_out"])
    np.testing.assert_allclose(np.concatenate([first["out"], second["out"]], 2), whole["out"], rtol=0, atol=1e-14)
    np.testing.assert_array_equal(second["state_out"], whole["state_out"])
    np.testing.assert_array_equal(whole["state_out"], x[:, :, 16 - (W - 1):])


def test_conv_token_by_token_equals_whole():
    r = _rng(8)
    x, w, b = r.normal(size=(2, 3, 9)), r.normal(size=(3, 4)), r.normal(size=3)
    whole = cv.conv_fwd(x, w, b)["out"]
    state = np.zeros((2, 3, 3))
    for t in range(9):
        o, state = cv.conv_step(state, x[:, :, t], w, b)
        np.testing.assert_allclose(o, whole[:, :, t], rtol=0, atol=1e-14)


@pytest.mark.parametrize("silu", [False, True])
def test_conv_gradient_finite_differences(silu):
    r = _rng(9)
    x, w, b = r.normal(size=(2, 3, 8)), r.normal(size=(3, 4)), r.normal(size=3)
    st = r.normal(size=(2, 3, 3))
    G = r.normal(size=(2, 3, 8))
    g = cv.conv_bwd(x, w, G, b, st, silu)

    def loss(x_, w_, b_):
        return float(np.sum(cv.conv_fwd(x_, w_, b_, st, silu)["out"] * G))
    eps = 1e-6
    for name, arr, grad in (("x", x, g["dx"]), ("w", w, g["dw"]), ("b", b, g["dbias"])):
        for idx in np.ndindex(arr.shape):
            hi, lo = arr.copy(), arr.copy()
            hi[idx] += eps
            lo[idx] -= eps
            args_hi = {"x": (hi, w, b), "w": (x, hi, b), "b": (x, w, hi)}[name]
            args_lo = {"x": (lo, w, b), "w": (x, lo, b), "b": (x, w, lo)}[name]
            fd = (loss(*args_hi) - loss(*args_lo)) / (2 * eps)
            assert grad[idx] == pytest.approx(fd, rel=1e-6, abs=1e-8), (name, idx)


# ---------------------------------------------------------------- the layer ----------------
def _layer(seed, B=2, D=4, L=9, N=3, R=2, W=4):
    r = _rng(seed)
    return dict(x=r.normal(size=(B, D, L)), z=r.normal(size=(B, D, L)), conv_w=r.normal(size=(D, W)) * 0.5,
                conv_b=r.normal(size=D) * 0.2, W_x=r.normal(size=(R + 2 * N, D)) * 0.5,
                W_dt=r.normal(size=(D, R)) * 0.5, dt_bias=r.normal(size=D) * 0.3,
                A=-np.abs(r.normal(size=(D, N))) - 0.2, Dskip=r.normal(size=D))


def test_layer_reduces_to_scan_with_hand_built_projections():
    """Projections that pick single channels: B, C and Delta become known functions of u."""
    B_, D, L, N, R = 2, 4, 11, 2, 1
    r = _rng(21)
    p = _layer(21, B_, D, L, N, R)
    # identity conv without bias: v = x, u = SiLU(x)
    p["conv_w"] = np.zeros((D, 4))
    p["conv_w"][:, 3] = 1.0
    p["conv_b"] = np.zeros(D)
    W_x = np.zeros((R + 2 * N, D))
    W_x[0, 0] = 1.0                    # r    = u[channel 0]
    W_x[1, 1], W_x[2, 2] = 2.0, -1.0   # B    = (2 u[1], -u[2])
    W_x[3, 3], W_x[4, 0] = 0.5, 1.5    # C    = (0.5 u[3], 1.5 u[0])
    p["W_x"] = W_x
    p["W_dt"] = r.normal(size=(D, R))  # delta_raw[d] = W_dt[d,0] * u[0]
    got = inn.inner_fwd(**p)
    u = p["x"] / (1.0 + np.exp(-p["x"]))
    Bm = np.stack([2.0 * u[:, 1], -u[:, 2]], axis=1)
    Cm = np.stack([0.5 * u[:, 3], 1.5 * u[:, 0]], axis=1)
    delta_raw = p["W_dt"][None, :, 0, None] * u[:, None, 0, :]
    ref = orc.scan_fwd(u, delta_raw, p["A"], Bm, Cm, Dskip=p["Dskip"], z=p["z"], bias=p["dt_bias"], softplus=True)
    np.testing.assert_allclose(got["out"], ref["out"], rtol=1e-12, atol=1e-13)


def test_layer_low_rank_delta_is_two_linear_maps():
    """Section 3.6: delta_raw = W_dt (W_x[:R] u), i.e. rank R across channels at every step."""
    p = _layer(22, D=6, R=2)
    f = inn.inner_fwd(**p)
    for b in range(2):
        assert np.linalg.matrix_rank(f["delta_raw"][b]) == 2
        np.testing.assert_allclose(f["delta_raw"][b], p["W_dt"] @ p["W_x"][:2] @ f["u"][b], rtol=1e-12, atol=1e-13)


def test_layer_is_causal():
    p = _layer(23)
    base = inn.inner_fwd(**p)["out"]
    p2 = dict(p)
    p2["x"] = p["x"].copy()
    p2["x"][:, :, 5] += 0.3
    out2 = inn.inner_fwd(**p2)["out"]
    np.testing.assert_array_equal(out2[:, :, :5], base[:, :, :5])
    assert np.abs(out2[:, :, 5:] - base[:, :, 5:]).max() > 1e-3


def test_layer_token_by_token_equals_whole_and_continues_a_prompt():
    p = _layer(28, L=12)
    whole = inn.inner_fwd(**p)
    w = {k: v for k, v in p.items() if k not in ("x", "z")}
    # from scratch
    h, cs = np.zeros((2, 4, 3)), np.zeros((2, 4, 3))
    for t in range(12):
        o, h, cs = inn.inner_step(h, cs, p["x"][:, :, t], p["z"][:, :, t], **w)
        np.testing.assert_allclose(o, whole["out"][:, :, t], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(h, whole["h_last"], rtol=1e-12, atol=1e-13)
    np.testing.assert_array_equal(cs, whole["conv_state"])
    # after a prompt of 7 tokens processed in parallel mode
    head = inn.inner_fwd(x=p["x"][:, :, :7], z=p["z"][:, :, :7], **w)
    h, cs = head["h_last"], head["conv_state"]
    for t in range(7, 12):
        o, h, cs = inn.inner_step(h, cs, p["x"][:, :, t], p["z"][:, :, t], **w)
        np.testing.assert_allclose(o, whole["out"][:, :, t], rtol=1e-12, atol=1e-13)


def test_layer_gradient_finite_differences():
    p = _layer(24)
    G = _rng(25).normal(size=p["x"].shape)
    g = inn.inner_bwd(dout=G, **p)
    names = {"x": "dx", "z": "dz", "conv_w": "dconv_w", "conv_b": "dconv_b", "W_x": "dW_x", "W_dt": "dW_dt",
             "dt_bias": "ddt_bias", "A": "dA", "Dskip": "dD"}
    assert set(g) == set(names.values())
    eps = 1e-6
    r = _rng(26)
    for name, gname in names.items():
        arr = p[name]
        assert g[gname].shape == arr.shape
        # a random direction over the whole tensor and three single coordinates
        probes = [r.normal(size=arr.shape)]
        for _ in range(3):
            e = np.zeros(arr.shape)
            e[tuple(r.integers(0, s) for s in arr.shape)] = 1.0
            probes.append(e)
        for v in probes:
            hi, lo = dict(p), dict(p)
            hi[name], lo[name] = arr + eps * v, arr - eps * v
            fd = (np.sum(inn.inner_fwd(**hi)["out"] * G) - np.sum(inn.inner_fwd(**lo)["out"] * G)) / (2 * eps)
            assert float(np.sum(g[gname] * v)) == pytest.approx(fd, rel=2e-6, abs=1e-8), name


def test_layer_rounding_hook_is_applied_at_the_three_stored_intermediates():
    from paper_2312_00752_amd.workloads import round_to_bf16
    p = _layer(27)
    f = inn.inner_fwd(rnd=lambda a: round_to_bf16(a).astype(np.float64), **p)
    for k in ("u", "P", "delta_raw"):
        np.testing.assert_array_equal(f[k], round_to_bf16(f[k]).astype(np.float64))
    exact = inn.inner_fwd(**p)
    assert 0 < np.abs(f["out"] - exact["out"]).max() < 0.2 * np.abs(exact["out"]).max()
