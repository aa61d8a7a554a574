"""The layer's projection products (ss_proj_gemm) against float64 matrix products on the CPU.

The shapes are the six products of the layer (Algorithm 2 with the projections of Sections 3.2
and 3.6, and their gradients) at sizes that span several tiles of every kernel, on the
matrix-core kernels, on the general kernel (forced, float32 operands, sizes that fit no tile) and
with strides that are not the dense ones.
"""
import pytest
import torch

from paper_2312_00752_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _rand(shape, dtype, seed):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(shape, generator=g) * 0.5).to(dtype).to(DEV)


def _check(A, Bm, C0, trans_a, trans_b, accumulate, general, c_dtype, workspace=None):
    """Operands on the GPU (views keep their strides); compare with the float64 product of the same (rounded) operands."""
    a64 = A.cpu().double().transpose(-1, -2) if trans_a else A.cpu().double()
    b64 = Bm.cpu().double().transpose(-1, -2) if trans_b else Bm.cpu().double()
    ref = torch.matmul(a64, b64)
    C = (C0.clone() if C0 is not None else torch.zeros(ref.shape, device=DEV)).to(c_dtype)
    if accumulate:
        ref = ref + C.cpu().double()
    else:
        C.fill_(float("nan"))   # every element must be written
    B.ss_proj_gemm(A, Bm, C, trans_a=trans_a, trans_b=trans_b, accumulate=accumulate, general=general, workspace=workspace)
    torch.cuda.synchronize()
    got = C.cpu().double()
    assert torch.isfinite(got).all()
    scale = ref.abs().max().item()
    # float32 accumulation of K products of O(1) terms; a bf16 result is rounded once (2^-9 relative)
    tol = 2e-2 if c_dtype == torch.bfloat16 else (1e-5 if A.dtype == torch.float32 else 1e-4)
    err = (got - ref).abs().max().item() / scale
    assert err <= tol, (err, tol)
    if c_dtype == torch.bfloat16:   # element-wise: within one rounding of the exact value
        assert ((got - ref).abs() <= 2.0 ** -8 * ref.abs() + 1e-3 * scale).all()


# (name, batch, D, L, R, Mx)
SHAPES = [("several_tiles", 2, 512, 256, 64, 96), ("headline_ranks", 1, 256, 256, 128, 160)]


@pytest.mark.parametrize("general", [False, True])
@pytest.mark.parametrize("name,nb,D,L,R,Mx", SHAPES)
def test_layer_products_bf16(name, nb, D, L, R, Mx, general):
    bf = torch.bfloat16
    u = _rand((nb, D, L), bf, 1)
    P = _rand((nb, Mx, L), bf, 2)
    W_x = _rand((Mx, D), bf, 3)
    W_dt = _rand((D, R), bf, 4)
    W_dtT = W_dt.t().contiguous()
    W_xT = W_x.t().contiguous()
    r = P[:, :R]                                   # rows of a larger matrix: batch stride Mx * L
    # [r;B;C] = W_x u            (few rows out, contraction over the rows of u)
    _check(W_x, u, None, False, False, False, general, bf)
    # dr = W_dt^T ddelta          (from a transposed copy of W_dt, as the layer makes one)
    _check(W_dtT, u, None, False, False, False, general, bf)
    # delta = W_dt r              (many rows out, short contraction)
    _check(W_dt, r, None, False, False, False, general, bf)
    # du += W_x^T dP              (accumulating, from a transposed copy of W_x)
    _check(W_xT, P, _rand((nb, D, L), bf, 5), False, False, True, general, bf)
    # dW_dt partials = ddelta r^T (both contiguous along the contraction index, float32 out)
    _check(u, r, None, False, True, False, general, torch.float32)
    # dW_x partials = dP u^T
    _check(P, u, None, False, True, False, general, torch.float32)


@pytest.mark.parametrize("nb,D,L,Mx", [(2, 4096, 256, 96), (1, 4608, 192, 160), (3, 1024, 128, 16)])
def test_split_contraction_with_workspace(nb, D, L, Mx):
    """[r;B;C] = W_x u with few column tiles: with a workspace the contraction is split over two workgroups per
    tile (D >= 4096, a multiple of 512), and the sum of the two float32 shares meets the same bounds.  A workspace that is
    too small, or a contraction that does not divide, silently runs unsplit."""
    bf = torch.bfloat16
    u = _rand((nb, D, L), bf, 11)
    W_x = _rand((Mx, D), bf, 12)
    C = torch.empty((nb, Mx, L), dtype=bf, device=DEV)
    need = B.ss_proj_gemm_workspace_bytes(C)
    assert need == 2 * nb * Mx * L * 4
    ws = torch.full((need,), 0xFF, dtype=torch.uint8, device=DEV)     # NaN patterns: every share must be written before it is read
    _check(W_x, u, None, False, False, False, False, bf, workspace=ws)
    _check(W_x, u, None, False, False, False, False, bf, workspace=ws[:need // 2])
    # rows of a wider result (row pitch and batch stride of the caller's)
    wide = torch.zeros((nb, Mx + 32, L + 64), dtype=bf, device=DEV)
    view = wide[:, :Mx, :L]
    B.ss_proj_gemm(W_x, u, view, workspace=ws)
    torch.cuda.synchronize()
    ref = torch.matmul(W_x.cpu().double(), u.cpu().double())
    assert ((view.cpu().double() - ref).abs() <= 2.0 ** -8 * ref.abs() + 1e-3 * ref.abs().max()).all()
    assert (wide[:, Mx:].abs().max() == 0) and (wide[:, :, L:].abs().max() == 0)   # nothing outside the result


def test_transposed_operands_and_odd_sizes():
    """Strides that only the general kernel takes: stored-transposed first operand, sizes off every tile."""
    bf = torch.bfloat16
    for dtype in (bf, torch.float32):
        A = _rand((3, 70, 37), dtype, 6)           # stored (K, M)
        Bm = _rand((3, 70, 45), dtype, 7)
        _check(A, Bm, None, True, False, False, False, dtype)
        W = _rand((45, 70), dtype, 8)              # shared, stored (N, K)
        _check(A, W, _rand((3, 37, 45), dtype, 9), True, True, True, False, dtype)
    # the per-token products of the decode path: (B, D) x (D, Mx)^T and (B, R) x (R, D)^T
    u_t = _rand((5, 96), bf, 10)
    W_x = _rand((40, 96), bf, 11)
    _check(u_t, W_x, None, False, True, False, False, bf)


def test_float32_layer_products():
    f32 = torch.float32
    u = _rand((2, 128, 192), f32, 12)
    W = _rand((48, 128), f32, 13)
    _check(W, u, None, False, False, False, False, f32)
    _check(u, _rand((2, 48, 192), f32, 14), None, False, True, False, False, f32)


def test_empty_and_rejections():
    bf = torch.bfloat16
    A = torch.zeros((4, 8), dtype=bf, device=DEV)
    C = torch.full((4, 4), 7.0, dtype=bf, device=DEV)
    # K = 0: an empty sum
    B.ss_proj_gemm(A[:, :0], torch.zeros((0, 4), dtype=bf, device=DEV), C)
    torch.cuda.synchronize()
    assert (C == 0).all()
    with pytest.raises(ValueError):
        B.ss_proj_gemm(A, torch.zeros((9, 4), dtype=bf, device=DEV), C)
