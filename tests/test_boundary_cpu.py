"""Boundary checks that need no GPU: the library loads, exports every declared symbol,
and rejects bad arguments on the host before any device call."""
import ctypes
import os
import re

import pytest

from paper_2312_00752_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000001000  # a non-null, 4096-byte aligned address that is never dereferenced


def test_library_exports_every_declared_symbol():
    names = set()
    inc = os.path.join(ROOT, "include")
    for fn in sorted(os.listdir(inc)):
        hdr = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, fn)).read(), flags=re.S)
        names |= set(re.findall(r"\b(ss_[a-z_]+)\s*\(", hdr))
    assert {"ss_scan_fwd", "ss_scan_bwd", "ss_step", "ss_workspace_bytes", "ss_strerror", "ss_version",
            "ss_conv_fwd", "ss_conv_bwd", "ss_conv_step", "ss_layer_fwd", "ss_layer_bwd", "ss_layer_step",
            "ss_layer_saved_bytes", "ss_layer_scratch_bytes", "ss_layer_step_scratch_bytes", "ss_proj_gemm",
            "ss_proj_gemm_workspace_bytes"} <= names
    lib = B.lib()
    for n in names:
        assert hasattr(lib, n), n
    assert B.ss_version() >= 100
    assert B.ss_strerror(0) == "success"
    for code in range(-7, 0):
        assert B.ss_strerror(code) not in ("", "success", "unknown error code")


def test_struct_layout_matches_header():
    assert ctypes.sizeof(B.FwdParams) == 6 * 4 + 13 * 8
    assert ctypes.sizeof(B.BwdParams) == ctypes.sizeof(B.FwdParams) + 11 * 8
    assert ctypes.sizeof(B.StepParams) == 5 * 4 + 4 + 10 * 8
    assert B.SS_CHECKPOINT_STEPS == 16 and B.SS_MAX_DSTATE == 256


def _good_fwd():
    p = B.FwdParams()
    p.batch, p.dim, p.seqlen, p.dstate = 2, 64, 128, 16
    p.io_dtype = B.SS_BF16
    for f in ("u", "delta", "Bmat", "Cmat", "A", "out"):
        setattr(p, f, FAKE)
    return p


def _fwd(p):
    return B.lib().ss_scan_fwd(ctypes.byref(p), None)


def test_forward_rejections():
    assert B.lib().ss_scan_fwd(None, None) == B.SS_ERR_NULL
    for f in ("u", "delta", "Bmat", "Cmat", "A", "out"):
        p = _good_fwd(); setattr(p, f, None)
        assert _fwd(p) == B.SS_ERR_NULL, f
    for f, v in (("batch", 0), ("dim", 0), ("dstate", 0), ("seqlen", -1), ("batch", -3)):
        p = _good_fwd(); setattr(p, f, v)
        assert _fwd(p) == B.SS_ERR_SHAPE, f
    p = _good_fwd(); p.dstate = 257
    assert _fwd(p) == B.SS_ERR_UNSUPPORTED
    p = _good_fwd(); p.io_dtype = 2
    assert _fwd(p) == B.SS_ERR_UNSUPPORTED
    p = _good_fwd(); p.flags = 1 << 20
    assert _fwd(p) == B.SS_ERR_UNSUPPORTED
    for flag, f in ((B.SS_HAS_Z, "z"), (B.SS_HAS_D, "Dskip"), (B.SS_HAS_DELTA_BIAS, "delta_bias"),
                    (B.SS_HAS_H0, "h0"), (B.SS_WRITE_H_LAST, "h_last")):
        p = _good_fwd(); p.flags = flag
        assert _fwd(p) == B.SS_ERR_NULL, f
    p = _good_fwd(); p.u = FAKE + 8
    assert _fwd(p) == B.SS_ERR_ALIGN
    p = _good_fwd(); p.A = FAKE + 2
    assert _fwd(p) == B.SS_ERR_ALIGN
    # checkpoints requested without / with too small a workspace
    p = _good_fwd(); p.flags = B.SS_SAVE_FOR_BWD
    assert _fwd(p) == B.SS_ERR_WORKSPACE
    need = B.ss_workspace_bytes(2, 64, 128, 16, io_dtype=B.SS_BF16, has_z=False)
    p.workspace = FAKE; p.workspace_bytes = need - 1
    assert _fwd(p) == B.SS_ERR_WORKSPACE
    p.workspace = FAKE + 128; p.workspace_bytes = need
    assert _fwd(p) == B.SS_ERR_ALIGN


def test_workspace_size_formula():
    # the repacked copy of B and C that the forward kernels read: B * ceil16(N) * (L rounded up to 32) * 2 elements
    def staged(batch, seqlen, dstate, esz=4):
        return -(-batch * (-(-dstate // 16) * 16) * (-(-seqlen // 32) * 32) * 2 * esz // 256) * 256
    # 96 steps: too short for the sequence to be split across workgroups
    assert B.ss_workspace_bytes(2, 64, 96, 16, for_backward=False) == staged(2, 96, 16)
    need = B.ss_workspace_bytes(2, 64, 96, 16)
    rows, chunks = 2 * 64, 96 // B.SS_CHECKPOINT_STEPS
    assert need >= (chunks * rows * 16 + rows * 96 + rows * 16 + 2 * rows) * 4 + staged(2, 96, 16)
    assert B.ss_workspace_bytes(2, 64, 96, 16, io_dtype=B.SS_BF16) == need - rows * 96 * 2 - staged(2, 96, 16, 2)
    assert B.ss_workspace_bytes(2, 64, 96, 16, has_z=False) == need - rows * 96 * 4
    assert need % 256 == 0
    assert B.ss_workspace_bytes(2, 64, 97, 16) > need          # a ragged tail adds a chunk
    assert B.ss_workspace_bytes(1, 1, 0, 1) % 256 == 0
    # no copy for a time-invariant B or C
    assert B.ss_workspace_bytes(2, 64, 96, 16, for_backward=False, b_fixed=True) == 0
    # few rows and a long sequence: scratch for splitting L across workgroups, also for a plain forward
    assert B.ss_workspace_bytes(1, 256, 1 << 20, 16, for_backward=False) >= 100 * 256 * 17 * 4 + staged(1, 1 << 20, 16)
    assert B.ss_workspace_bytes(8, 4096, 2048, 16, for_backward=False) == staged(8, 2048, 16)  # two workgroups per compute unit: never split
    assert B.ss_workspace_bytes(8, 2048, 2048, 16, for_backward=False) > staged(8, 2048, 16)   # one row tile per compute unit: split
    assert B.ss_workspace_bytes(1, 1024, 1024, 16, for_backward=False) > staged(1, 1024, 16)   # few row tiles: split even when short
    assert B.ss_workspace_bytes(1, 256, 96, 16, for_backward=False) == staged(1, 96, 16)       # too short to split
    # a very long sequence is not cut into thousands of short segments: each workgroup has a fixed cost
    split = B.ss_workspace_bytes(1, 1024, 1 << 18, 16, for_backward=False) - staged(1, 1 << 18, 16)
    assert 0 < split <= 128 * 1024 * 17 * 4 + 512


def test_backward_rejections():
    q = B.BwdParams()
    q.fwd = _good_fwd()
    q.fwd.out = None                      # not needed by the backward call
    need = B.ss_workspace_bytes(2, 64, 128, 16)   # upper bound over dtypes and flags
    q.fwd.workspace = FAKE; q.fwd.workspace_bytes = need
    for f in ("dout", "du", "ddelta", "dB", "dC", "dA"):
        setattr(q, f, FAKE)
    bwd = lambda: B.lib().ss_scan_bwd(ctypes.byref(q), None)
    for f in ("dout", "du", "ddelta", "dB", "dC", "dA"):
        setattr(q, f, None)
        assert bwd() == B.SS_ERR_NULL, f
        setattr(q, f, FAKE)
    q.fwd.flags = B.SS_HAS_Z; q.fwd.z = FAKE
    assert bwd() == B.SS_ERR_NULL         # dz missing
    q.dz = FAKE; q.fwd.flags |= B.SS_HAS_D; q.fwd.Dskip = FAKE
    assert bwd() == B.SS_ERR_NULL         # dD missing
    q.dD = FAKE; q.fwd.flags |= B.SS_HAS_DELTA_BIAS; q.fwd.delta_bias = FAKE
    assert bwd() == B.SS_ERR_NULL         # ddelta_bias missing
    exact = B.ss_workspace_bytes(2, 64, 128, 16, io_dtype=B.SS_BF16, has_z=True)
    q.ddelta_bias = FAKE; q.fwd.workspace_bytes = exact - 256
    assert bwd() == B.SS_ERR_WORKSPACE
    q.fwd.workspace_bytes = exact; q.du = FAKE + 4
    assert bwd() == B.SS_ERR_ALIGN
    assert B.lib().ss_scan_bwd(None, None) == B.SS_ERR_NULL


def test_step_rejections():
    def good():
        p = B.StepParams()
        p.batch, p.dim, p.dstate, p.io_dtype = 4, 32, 16, B.SS_F32
        for f in ("h", "u_t", "delta_t", "B_t", "C_t", "A", "out_t"):
            setattr(p, f, FAKE)
        return p
    step = lambda p: B.lib().ss_step(ctypes.byref(p), None)
    assert B.lib().ss_step(None, None) == B.SS_ERR_NULL
    for f in ("h", "u_t", "delta_t", "B_t", "C_t", "A", "out_t"):
        p = good(); setattr(p, f, None)
        assert step(p) == B.SS_ERR_NULL, f
    p = good(); p.dstate = 0
    assert step(p) == B.SS_ERR_SHAPE
    p = good(); p.dstate = 257
    assert step(p) == B.SS_ERR_UNSUPPORTED
    p = good(); p.flags = B.SS_HAS_H0
    assert step(p) == B.SS_ERR_UNSUPPORTED
    p = good(); p.flags = B.SS_HAS_Z
    assert step(p) == B.SS_ERR_NULL
    p = good(); p.h = FAKE + 4
    assert step(p) == B.SS_ERR_ALIGN


def test_python_wrappers_refuse_cpu_tensors():
    import torch
    u = torch.zeros(1, 4, 8)
    A = torch.zeros(4, 2)
    Bm = torch.zeros(1, 2, 8)
    with pytest.raises(ValueError):
        B.ss_scan_fwd(u, u, A, Bm, Bm)


# ---------------------------------------------------------------- short convolution
def _good_conv():
    p = B.ConvParams()
    p.batch, p.dim, p.seqlen, p.width = 2, 64, 128, 4
    p.io_dtype = B.SS_BF16
    p.flags = B.SS_CONV_SILU | B.SS_CONV_HAS_BIAS
    for f in ("x", "w", "bias", "out"):
        setattr(p, f, FAKE)
    return p


def test_conv_struct_layout_and_rejections():
    assert ctypes.sizeof(B.ConvParams) == 6 * 4 + 6 * 8
    assert ctypes.sizeof(B.ConvBwdParams) == ctypes.sizeof(B.ConvParams) + 4 * 8
    assert ctypes.sizeof(B.ConvStepParams) == 5 * 4 + 4 + 5 * 8
    fwd = lambda p: B.lib().ss_conv_fwd(ctypes.byref(p), None)
    assert B.lib().ss_conv_fwd(None, None) == B.SS_ERR_NULL
    for f in ("x", "w", "bias", "out"):
        p = _good_conv(); setattr(p, f, None)
        assert fwd(p) == B.SS_ERR_NULL, f
    for f, v in (("batch", 0), ("dim", 0), ("seqlen", -1), ("width", 0)):
        p = _good_conv(); setattr(p, f, v)
        assert fwd(p) == B.SS_ERR_SHAPE, f
    p = _good_conv(); p.width = 5
    assert fwd(p) == B.SS_ERR_UNSUPPORTED
    p = _good_conv(); p.flags = 16
    assert fwd(p) == B.SS_ERR_UNSUPPORTED
    p = _good_conv(); p.io_dtype = 7
    assert fwd(p) == B.SS_ERR_UNSUPPORTED
    p = _good_conv(); p.x = FAKE + 8
    assert fwd(p) == B.SS_ERR_ALIGN
    p = _good_conv(); p.flags |= B.SS_CONV_HAS_STATE
    assert fwd(p) == B.SS_ERR_NULL
    p = _good_conv(); p.flags |= B.SS_CONV_WRITE_STATE
    assert fwd(p) == B.SS_ERR_NULL
    q = B.ConvBwdParams(); q.fwd = _good_conv()
    bwd = lambda q: B.lib().ss_conv_bwd(ctypes.byref(q), None)
    assert bwd(q) == B.SS_ERR_NULL           # dw missing
    q.dw = FAKE
    assert bwd(q) == B.SS_ERR_NULL           # dbias missing although a bias is given
    q.dbias = FAKE
    assert bwd(q) == B.SS_ERR_NULL           # dout / dx missing
    s = B.ConvStepParams()
    s.batch, s.dim, s.width, s.io_dtype = 2, 8, 4, B.SS_F32
    assert B.lib().ss_conv_step(ctypes.byref(s), None) == B.SS_ERR_NULL
    s.width = 9
    assert B.lib().ss_conv_step(ctypes.byref(s), None) == B.SS_ERR_UNSUPPORTED


# ---------------------------------------------------------------- the layer
def _good_layer():
    p = B.LayerParams()
    p.batch, p.dim, p.seqlen, p.dstate, p.dt_rank, p.conv_width = 2, 64, 128, 16, 4, 4
    p.io_dtype = B.SS_BF16
    for f in ("x", "z", "conv_w", "conv_b", "W_x", "W_dt", "dt_bias", "A", "Dskip", "out", "scratch"):
        setattr(p, f, FAKE)
    p.scratch_bytes = 1 << 30
    return p


def test_layer_struct_layout_sizes_and_rejections():
    assert ctypes.sizeof(B.LayerParams) == 8 * 4 + 16 * 8
    assert ctypes.sizeof(B.LayerBwdParams) == ctypes.sizeof(B.LayerParams) + 10 * 8
    assert ctypes.sizeof(B.LayerStepParams) == 7 * 4 + 4 + 14 * 8
    saved = B.ss_layer_saved_bytes(8, 4096, 2048, 16, 128)
    # [r;B;C] in bf16 plus the scan's own workspace
    assert saved >= 8 * 160 * 2048 * 2 + B.ss_workspace_bytes(8, 4096, 2048, 16, True, B.SS_BF16, True)
    assert saved < 1.02 * (8 * 160 * 2048 * 2 + B.ss_workspace_bytes(8, 4096, 2048, 16, True, B.SS_BF16, True))
    assert B.ss_layer_scratch_bytes(8, 4096, 2048, 16, 128, for_backward=False) >= 2 * 8 * 4096 * 2048 * 2
    assert B.ss_layer_scratch_bytes(8, 4096, 2048, 16, 128, for_backward=True) >= 4 * 8 * 4096 * 2048 * 2
    fwd = lambda p: B.lib().ss_layer_fwd(ctypes.byref(p), None)
    assert B.lib().ss_layer_fwd(None, None) == B.SS_ERR_NULL
    for f in ("x", "z", "conv_w", "conv_b", "W_x", "W_dt", "dt_bias", "A", "Dskip", "out"):
        p = _good_layer(); setattr(p, f, None)
        assert fwd(p) == B.SS_ERR_NULL, f
    for f, v in (("batch", 0), ("dim", 0), ("seqlen", 0), ("dstate", 0), ("dt_rank", 0), ("conv_width", 0)):
        p = _good_layer(); setattr(p, f, v)
        assert fwd(p) == B.SS_ERR_SHAPE, f
    p = _good_layer(); p.dstate = 257
    assert fwd(p) == B.SS_ERR_UNSUPPORTED
    p = _good_layer(); p.flags = 1
    assert fwd(p) == B.SS_ERR_UNSUPPORTED
    p = _good_layer(); p.scratch_bytes = 1000
    assert fwd(p) == B.SS_ERR_WORKSPACE
    p = _good_layer(); p.scratch = None
    assert fwd(p) == B.SS_ERR_WORKSPACE
    p = _good_layer(); p.saved = FAKE; p.saved_bytes = 10
    assert fwd(p) == B.SS_ERR_WORKSPACE
    p = _good_layer(); p.x = FAKE + 4
    assert fwd(p) == B.SS_ERR_ALIGN
    q = B.LayerBwdParams(); q.fwd = _good_layer()
    assert B.lib().ss_layer_bwd(ctypes.byref(q), None) == B.SS_ERR_WORKSPACE   # nothing saved
    s = B.LayerStepParams()
    s.batch, s.dim, s.dstate, s.dt_rank, s.conv_width, s.io_dtype = 2, 8, 4, 2, 4, B.SS_F32
    assert B.lib().ss_layer_step(ctypes.byref(s), None) == B.SS_ERR_NULL
    assert B.ss_strerror(B.SS_ERR_BACKEND) not in ("", "unknown error code")


def test_time_invariant_bc_flags():
    # partial sums for the (D,N) gradients are added to the workspace, and the sequence is never split
    base = B.ss_workspace_bytes(1, 256, 1 << 16, 16, True, B.SS_F32, True)
    fixed = B.ss_workspace_bytes(1, 256, 1 << 16, 16, True, B.SS_F32, True, b_fixed=True, c_fixed=True)
    assert fixed != base
    assert B.ss_workspace_bytes(1, 256, 1 << 16, 16, False, B.SS_F32, True) > 0
    assert B.ss_workspace_bytes(1, 256, 1 << 16, 16, False, B.SS_F32, True, b_fixed=True) == 0
    small = B.ss_workspace_bytes(2, 64, 96, 16, True, B.SS_BF16, True)
    # ... and there is no repacked copy of B and C (2 * 16 * 96 * 2 bf16 values)
    assert B.ss_workspace_bytes(2, 64, 96, 16, True, B.SS_BF16, True, b_fixed=True) == small + 2 * 64 * 16 * 4 - 2 * 16 * 96 * 2 * 2
    # a (D,N) float32 parameter needs only 4-byte alignment
    p = _good_fwd(); p.flags = B.SS_B_FIXED; p.Bmat = FAKE + 4
    assert _fwd(p) != B.SS_ERR_ALIGN
    p = _good_fwd(); p.Bmat = FAKE + 4
    assert _fwd(p) == B.SS_ERR_ALIGN


def test_headers_are_plain_c():
    """The boundary is a C ABI: every header must compile as C99 on its own."""
    import subprocess
    inc = os.path.join(ROOT, "include")
    for fn in sorted(os.listdir(inc)):
        r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c",
                            "-I", inc, os.path.join(inc, fn)], capture_output=True, text=True)
        assert r.returncode == 0, fn + "\n" + r.stderr


def test_complex_state_flag():
    # complex states count twice against the limit and exclude the exact zero-order hold
    p = _good_fwd(); p.flags = B.SS_COMPLEX_STATE | B.SS_EXACT_ZOH_B
    assert _fwd(p) == B.SS_ERR_UNSUPPORTED
    p = _good_fwd(); p.flags = B.SS_COMPLEX_STATE; p.dstate = 129
    assert _fwd(p) == B.SS_ERR_UNSUPPORTED
    # 16 complex states are two groups of 16 slots: checkpoints double
    one = B.ss_workspace_bytes(2, 64, 96, 16, True, B.SS_BF16, False)
    two = B.ss_workspace_bytes(2, 64, 96, 16, True, B.SS_BF16, False, complex_state=True)
    # (and the real variant alone carries the repacked copy of B and C: 2 * 16 * 96 * 2 bf16 values)
    assert two > one and two - one == (96 // 16) * 2 * 64 * 16 * 4 - 2 * 16 * 96 * 2 * 2


def test_static_scratch_forward_rejections():
    """ss_scan_fwd_static validates like ss_scan_fwd, refuses the backward-saving mode and
    problems whose scratch exceeds its fixed array -- all on the host, before any device call."""
    f = B.lib().ss_scan_fwd_static
    assert f(None, None) == B.SS_ERR_NULL
    p = _good_fwd(); p.u = None
    assert f(ctypes.byref(p), None) == B.SS_ERR_NULL
    p = _good_fwd(); p.batch = 0
    assert f(ctypes.byref(p), None) == B.SS_ERR_SHAPE
    p = _good_fwd(); p.out = FAKE + 2
    assert f(ctypes.byref(p), None) == B.SS_ERR_ALIGN
    p = _good_fwd(); p.flags = B.SS_SAVE_FOR_BWD
    assert f(ctypes.byref(p), None) == B.SS_ERR_UNSUPPORTED
    # float32 I/O, one batch entry, 2^20 steps: the repacked B and C alone are 128 MiB
    p = _good_fwd(); p.io_dtype = B.SS_F32; p.batch, p.dim, p.seqlen = 1, 256, 1 << 20
    assert B.ss_workspace_bytes(1, 256, 1 << 20, 16, for_backward=False, io_dtype=B.SS_F32, has_z=False) > B.SS_STATIC_SCRATCH_BYTES
    assert f(ctypes.byref(p), None) == B.SS_ERR_WORKSPACE
    hdr = open(os.path.join(ROOT, "include", "ss_scan.h")).read()
    assert "#define SS_STATIC_SCRATCH_BYTES (64u << 20)" in hdr


def test_projection_product_rejections():
    g = B.GemmParams()
    call = lambda: B.lib().ss_proj_gemm(ctypes.byref(g), None)
    assert B.lib().ss_proj_gemm(None, None) == B.SS_ERR_NULL
    g.M, g.N, g.K, g.batch, g.io_dtype = 4, 4, 4, 1, B.SS_BF16
    assert call() == B.SS_ERR_NULL                      # no operands
    g.A = g.B = g.C = FAKE
    g.M = -1
    assert call() == B.SS_ERR_SHAPE
    g.M = 4; g.io_dtype = 7
    assert call() == B.SS_ERR_UNSUPPORTED
    g.io_dtype = B.SS_BF16; g.flags = 8
    assert call() == B.SS_ERR_UNSUPPORTED               # unknown flag
    g.flags = 0; g.batch = 70000
    assert call() == B.SS_ERR_UNSUPPORTED               # more batch entries than a launch takes
    g.batch = 0
    assert call() == B.SS_OK                            # nothing to do
    size = B.lib().ss_proj_gemm_workspace_bytes
    assert size(None) == 0
    g.M, g.N, g.batch = 160, 2048, 8
    assert size(ctypes.byref(g)) == 2 * 8 * 160 * 2048 * 4   # two float32 shares of the result
    g.N = -1
    assert size(ctypes.byref(g)) == 0


def test_skewed_allocation_helper():
    """Tensors for one call carved from one allocation: right shapes, contiguous, 256-byte aligned starts,
    each 65 KiB further into the interleave than the one before, no overlap."""
    import torch
    ts = B.empty_channel_skewed(3, (2, 5, 64), torch.bfloat16, "cpu")
    assert len(ts) == 3 and all(t.shape == (2, 5, 64) and t.dtype == torch.bfloat16 and t.is_contiguous() for t in ts)
    nbytes = 2 * 5 * 64 * 2
    starts = [t.data_ptr() for t in ts]
    assert all((b - a) == (nbytes + 255) // 256 * 256 + B.CHANNEL_SKEW_BYTES for a, b in zip(starts, starts[1:]))
    assert all((s_ - starts[0]) % 256 == 0 for s_ in starts)
    for i, t in enumerate(ts):
        t.fill_(float(i + 1))
    assert [float(t.float().min()) for t in ts] == [1.0, 2.0, 3.0] and [float(t.float().max()) for t in ts] == [1.0, 2.0, 3.0]
    assert B.empty_channel_skewed(0, (4,), torch.float32, "cpu") == []
