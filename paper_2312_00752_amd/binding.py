"""Thin ctypes binding of the C-ABI library declared in ``include/ss_scan.h``, ``include/ss_conv.h`` and ``include/ss_layer.h``.

Argument marshalling only: every step of the path runs in the library's HIP kernels.
PyTorch appears here solely as the owner of device memory and streams.  The library must
have been built (``python -m paper_2312_00752_amd.build``); loading fails loudly if it
has not been.
"""
import ctypes
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libss_scan.so")

SS_F32, SS_BF16 = 0, 1
SS_DELTA_SOFTPLUS, SS_HAS_DELTA_BIAS, SS_HAS_D, SS_HAS_Z = 1, 2, 4, 8
SS_HAS_H0, SS_WRITE_H_LAST, SS_SAVE_FOR_BWD, SS_EXACT_ZOH_B = 16, 32, 64, 128
SS_B_FIXED, SS_C_FIXED, SS_COMPLEX_STATE = 256, 512, 1024
SS_OK, SS_ERR_NULL, SS_ERR_SHAPE, SS_ERR_UNSUPPORTED = 0, -1, -2, -3
SS_ERR_ALIGN, SS_ERR_WORKSPACE, SS_ERR_LAUNCH = -4, -5, -6
SS_MAX_DSTATE = 256
SS_CHECKPOINT_STEPS = 16
SS_STATIC_SCRATCH_BYTES = 64 << 20

_vp = ctypes.c_void_p


class FwdParams(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("dim", ctypes.c_int32), ("seqlen", ctypes.c_int32),
                ("dstate", ctypes.c_int32), ("io_dtype", ctypes.c_int32), ("flags", ctypes.c_uint32),
                ("u", _vp), ("delta", _vp), ("z", _vp), ("Bmat", _vp), ("Cmat", _vp),
                ("A", _vp), ("Dskip", _vp), ("delta_bias", _vp), ("h0", _vp),
                ("out", _vp), ("h_last", _vp), ("workspace", _vp), ("workspace_bytes", ctypes.c_size_t)]


class BwdParams(ctypes.Structure):
    _fields_ = [("fwd", FwdParams), ("dout", _vp), ("dh_last", _vp),
                ("du", _vp), ("ddelta", _vp), ("dz", _vp), ("dB", _vp), ("dC", _vp),
                ("dA", _vp), ("dD", _vp), ("ddelta_bias", _vp), ("dh0", _vp)]


class StepParams(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("dim", ctypes.c_int32), ("dstate", ctypes.c_int32),
                ("io_dtype", ctypes.c_int32), ("flags", ctypes.c_uint32),
                ("h", _vp), ("u_t", _vp), ("delta_t", _vp), ("z_t", _vp), ("B_t", _vp), ("C_t", _vp),
                ("A", _vp), ("Dskip", _vp), ("delta_bias", _vp), ("out_t", _vp)]


class ConvParams(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("dim", ctypes.c_int32), ("seqlen", ctypes.c_int32),
                ("width", ctypes.c_int32), ("io_dtype", ctypes.c_int32), ("flags", ctypes.c_uint32),
                ("x", _vp), ("w", _vp), ("bias", _vp), ("state_in", _vp), ("out", _vp), ("state_out", _vp)]


class ConvBwdParams(ctypes.Structure):
    _fields_ = [("fwd", ConvParams), ("dout", _vp), ("dx", _vp), ("dw", _vp), ("dbias", _vp)]


class ConvStepParams(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("dim", ctypes.c_int32), ("width", ctypes.c_int32),
                ("io_dtype", ctypes.c_int32), ("flags", ctypes.c_uint32),
                ("state", _vp), ("x_t", _vp), ("w", _vp), ("bias", _vp), ("out_t", _vp)]


class LayerParams(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("dim", ctypes.c_int32), ("seqlen", ctypes.c_int32),
                ("dstate", ctypes.c_int32), ("dt_rank", ctypes.c_int32), ("conv_width", ctypes.c_int32),
                ("io_dtype", ctypes.c_int32), ("flags", ctypes.c_uint32),
                ("x", _vp), ("z", _vp), ("conv_w", _vp), ("conv_b", _vp), ("W_x", _vp), ("W_dt", _vp),
                ("dt_bias", _vp), ("A", _vp), ("Dskip", _vp), ("out", _vp),
                ("h_last", _vp), ("conv_state", _vp),
                ("saved", _vp), ("saved_bytes", ctypes.c_size_t),
                ("scratch", _vp), ("scratch_bytes", ctypes.c_size_t)]


class LayerBwdParams(ctypes.Structure):
    _fields_ = [("fwd", LayerParams), ("dout", _vp), ("dx", _vp), ("dz", _vp),
                ("dconv_w", _vp), ("dconv_b", _vp), ("dW_x", _vp), ("dW_dt", _vp),
                ("ddt_bias", _vp), ("dA", _vp), ("dD", _vp)]


class LayerStepParams(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("dim", ctypes.c_int32), ("dstate", ctypes.c_int32),
                ("dt_rank", ctypes.c_int32), ("conv_width", ctypes.c_int32), ("io_dtype", ctypes.c_int32),
                ("flags", ctypes.c_uint32),
                ("h", _vp), ("conv_state", _vp), ("x_t", _vp), ("z_t", _vp), ("conv_w", _vp), ("conv_b", _vp),
                ("W_x", _vp), ("W_dt", _vp), ("dt_bias", _vp), ("A", _vp), ("Dskip", _vp), ("out_t", _vp),
                ("scratch", _vp), ("scratch_bytes", ctypes.c_size_t)]


class GemmParams(ctypes.Structure):
    _fields_ = [("M", ctypes.c_int32), ("N", ctypes.c_int32), ("K", ctypes.c_int32), ("batch", ctypes.c_int32),
                ("io_dtype", ctypes.c_int32), ("flags", ctypes.c_uint32),
                ("A", _vp), ("a_m", ctypes.c_int64), ("a_k", ctypes.c_int64), ("a_batch", ctypes.c_int64),
                ("B", _vp), ("b_k", ctypes.c_int64), ("b_n", ctypes.c_int64), ("b_batch", ctypes.c_int64),
                ("C", _vp), ("ldc", ctypes.c_int64), ("c_batch", ctypes.c_int64),
                ("workspace", _vp), ("workspace_bytes", ctypes.c_size_t)]


SS_GEMM_C_FLOAT, SS_GEMM_ACCUMULATE, SS_GEMM_GENERAL = 1, 2, 4
SS_ERR_BACKEND = -7
SS_CONV_SILU, SS_CONV_HAS_BIAS, SS_CONV_HAS_STATE, SS_CONV_WRITE_STATE = 1, 2, 4, 8
SS_CONV_MAX_WIDTH = 4

_lib = None


def lib():
    """The loaded library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("%s is missing: build it with `python -m paper_2312_00752_amd.build`"
                               % LIB_PATH)
        l = ctypes.CDLL(LIB_PATH)
        l.ss_workspace_bytes.restype = ctypes.c_size_t
        l.ss_workspace_bytes.argtypes = [ctypes.POINTER(FwdParams), ctypes.c_int]
        l.ss_scan_fwd.restype = ctypes.c_int
        l.ss_scan_fwd.argtypes = [ctypes.POINTER(FwdParams), _vp]
        l.ss_scan_fwd_static.restype = ctypes.c_int
        l.ss_scan_fwd_static.argtypes = [ctypes.POINTER(FwdParams), _vp]
        l.ss_scan_bwd.restype = ctypes.c_int
        l.ss_scan_bwd.argtypes = [ctypes.POINTER(BwdParams), _vp]
        l.ss_step.restype = ctypes.c_int
        l.ss_step.argtypes = [ctypes.POINTER(StepParams), _vp]
        l.ss_conv_fwd.restype = ctypes.c_int
        l.ss_conv_fwd.argtypes = [ctypes.POINTER(ConvParams), _vp]
        l.ss_conv_bwd.restype = ctypes.c_int
        l.ss_conv_bwd.argtypes = [ctypes.POINTER(ConvBwdParams), _vp]
        l.ss_conv_step.restype = ctypes.c_int
        l.ss_conv_step.argtypes = [ctypes.POINTER(ConvStepParams), _vp]
        l.ss_layer_saved_bytes.restype = ctypes.c_size_t
        l.ss_layer_saved_bytes.argtypes = [ctypes.POINTER(LayerParams)]
        l.ss_layer_scratch_bytes.restype = ctypes.c_size_t
        l.ss_layer_scratch_bytes.argtypes = [ctypes.POINTER(LayerParams), ctypes.c_int]
        l.ss_layer_fwd.restype = ctypes.c_int
        l.ss_layer_fwd.argtypes = [ctypes.POINTER(LayerParams), _vp]
        l.ss_layer_bwd.restype = ctypes.c_int
        l.ss_layer_bwd.argtypes = [ctypes.POINTER(LayerBwdParams), _vp]
        l.ss_layer_step_scratch_bytes.restype = ctypes.c_size_t
        l.ss_layer_step_scratch_bytes.argtypes = [ctypes.POINTER(LayerStepParams)]
        l.ss_layer_step.restype = ctypes.c_int
        l.ss_layer_step.argtypes = [ctypes.POINTER(LayerStepParams), _vp]
        l.ss_strerror.restype = ctypes.c_char_p
        l.ss_proj_gemm.argtypes = [ctypes.POINTER(GemmParams), _vp]
        l.ss_proj_gemm.restype = ctypes.c_int
        l.ss_proj_gemm_workspace_bytes.argtypes = [ctypes.POINTER(GemmParams)]
        l.ss_proj_gemm_workspace_bytes.restype = ctypes.c_size_t
        l.ss_strerror.argtypes = [ctypes.c_int]
        l.ss_version.restype = ctypes.c_int
        l.ss_version.argtypes = []
        _lib = l
    return _lib


class SsError(RuntimeError):
    def __init__(self, code):
        self.code = code
        super().__init__("ss_scan error %d: %s" % (code, ss_strerror(code)))


def ss_strerror(code):
    return lib().ss_strerror(int(code)).decode()


def ss_version():
    return int(lib().ss_version())


# ---------------------------------------------------------------- tensor marshalling
def _io_code(t):
    import torch
    if t.dtype == torch.float32:
        return SS_F32
    if t.dtype == torch.bfloat16:
        return SS_BF16
    raise TypeError("io tensors must be float32 or bfloat16, got %s" % t.dtype)


def _ptr(t, dtype=None, shape=None, name="tensor"):
    """Device pointer of a dense CUDA tensor (or None)."""
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("%s must live on the GPU" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if dtype is not None and t.dtype != dtype:
        raise TypeError("%s must be %s, got %s" % (name, dtype, t.dtype))
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s must have shape %s, got %s" % (name, tuple(shape), tuple(t.shape)))
    return t.data_ptr()


CHANNEL_SKEW_BYTES = 66560   # 260 x 256


def empty_channel_skewed(n, shape, dtype, device):
    """``n`` uninitialised tensors of ``shape`` carved from ONE allocation, each starting 65 KiB (plus
    rounding to 256 bytes) after the end of the one before.

    Why: the scan kernels touch all of a call's (B,D,L) tensors at the same row and step at about the
    same time.  When a row is a large power of two of bytes (L = 2^20 float32: 4 MiB), the 64 rows of a
    workgroup already share one memory channel; if the tensors themselves also start at the same offset
    into the channels' interleave (separate large allocations do: each is aligned to its own large power
    of two), every access of the workgroup at that step queues on a single channel.  Placing the
    tensors at mutually skewed addresses takes the tensor-to-tensor part of that away (2^20-step
    float32 workload: 9.5 -> 7.6 ms forward + backward); shapes with short rows are unaffected.  The
    library cannot do this for tensors it is handed; callers that allocate them can."""
    import math
    import torch
    esz = torch.empty((), dtype=dtype).element_size()
    nbytes = int(math.prod(shape)) * esz
    pitch = (nbytes + 255) // 256 * 256 + CHANNEL_SKEW_BYTES
    pool = torch.empty(max(1, n * pitch), dtype=torch.uint8, device=device)
    return [pool[i * pitch: i * pitch + nbytes].view(dtype).view(tuple(shape)) for i in range(n)]


def _stream(stream):
    import torch
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _fwd_params(u, delta, A, Bmat, Cmat, Dskip, z, delta_bias, h0, delta_softplus, exact_zoh=False,
                complex_state=False):
    import torch
    f32 = torch.float32
    nb, nd, nl = u.shape
    nn = A.shape[1]
    io = u.dtype
    p = FwdParams()
    p.batch, p.dim, p.seqlen, p.dstate = nb, nd, nl, nn
    p.io_dtype = _io_code(u)
    flags = SS_COMPLEX_STATE if complex_state else 0
    # complex state: every complex array has a (re, im) axis right after the state axis
    c2 = (2,) if complex_state else ()
    p.u = _ptr(u, io, (nb, nd, nl), "u")
    p.delta = _ptr(delta, io, (nb, nd, nl), "delta")
    # a 2-D float32 (D,N) tensor is the time-invariant form of B / C (Algorithm 1)
    if Bmat.dim() == 2 + len(c2):
        p.Bmat = _ptr(Bmat, f32, (nd, nn) + c2, "Bmat")
        flags |= SS_B_FIXED
    else:
        p.Bmat = _ptr(Bmat, io, (nb, nn) + c2 + (nl,), "Bmat")
    if Cmat.dim() == 2 + len(c2):
        p.Cmat = _ptr(Cmat, f32, (nd, nn) + c2, "Cmat")
        flags |= SS_C_FIXED
    else:
        p.Cmat = _ptr(Cmat, io, (nb, nn) + c2 + (nl,), "Cmat")
    p.A = _ptr(A, f32, (nd, nn) + c2, "A")
    if z is not None:
        p.z = _ptr(z, io, (nb, nd, nl), "z")
        flags |= SS_HAS_Z
    if Dskip is not None:
        p.Dskip = _ptr(Dskip, f32, (nd,), "Dskip")
        flags |= SS_HAS_D
    if delta_bias is not None:
        p.delta_bias = _ptr(delta_bias, f32, (nd,), "delta_bias")
        flags |= SS_HAS_DELTA_BIAS
    if h0 is not None:
        p.h0 = _ptr(h0, f32, (nb, nd, nn) + c2, "h0")
        flags |= SS_HAS_H0
    if delta_softplus:
        flags |= SS_DELTA_SOFTPLUS
    if exact_zoh:
        flags |= SS_EXACT_ZOH_B
    p.flags = flags
    return p


def ss_workspace_bytes(batch, dim, seqlen, dstate, for_backward=True, io_dtype=SS_F32, has_z=True,
                       b_fixed=False, c_fixed=False, complex_state=False):
    """Workspace size; the defaults (float32 I/O, gate present) give an upper bound for selective B, C."""
    p = FwdParams()
    p.batch, p.dim, p.seqlen, p.dstate = batch, dim, seqlen, dstate
    p.io_dtype = io_dtype
    p.flags = ((SS_HAS_Z if has_z else 0) | (SS_B_FIXED if b_fixed else 0) | (SS_C_FIXED if c_fixed else 0)
               | (SS_COMPLEX_STATE if complex_state else 0))
    return int(lib().ss_workspace_bytes(ctypes.byref(p), int(bool(for_backward))))


def ss_scan_fwd(u, delta, A, Bmat, Cmat, Dskip=None, z=None, delta_bias=None, h0=None,
                delta_softplus=False, out=None, h_last=None, return_last_state=False,
                workspace=None, save_for_bwd=True, exact_zoh=False, complex_state=False, stream=None):
    """Enqueue the forward scan.  Returns (out, h_last or None).
    With ``complex_state`` A is (D,N,2), B and C (B,N,2,L), h0 / h_last (B,D,N,2): (re, im) pairs.

    ``workspace`` is a uint8 CUDA tensor of at least ``ss_workspace_bytes(...)`` bytes.  With
    ``save_for_bwd`` (the default when a workspace is given) the call leaves what
    ``ss_scan_bwd`` needs in it; without, the workspace only serves as scratch that lets
    a long sequence with few rows be split across workgroups."""
    import torch
    p = _fwd_params(u, delta, A, Bmat, Cmat, Dskip, z, delta_bias, h0, delta_softplus, exact_zoh, complex_state)
    state_shape = (p.batch, p.dim, p.dstate) + ((2,) if complex_state else ())
    if out is None:
        out = torch.empty_like(u)
    p.out = _ptr(out, u.dtype, u.shape, "out")
    if return_last_state or h_last is not None:
        if h_last is None:
            h_last = torch.empty(state_shape, dtype=torch.float32, device=u.device)
        p.h_last = _ptr(h_last, torch.float32, state_shape, "h_last")
        p.flags |= SS_WRITE_H_LAST
    if workspace is not None:
        p.workspace = _ptr(workspace, torch.uint8, None, "workspace")
        p.workspace_bytes = workspace.numel()
        if save_for_bwd:
            p.flags |= SS_SAVE_FOR_BWD
    rc = lib().ss_scan_fwd(ctypes.byref(p), _stream(stream))
    if rc != SS_OK:
        raise SsError(rc)
    return out, h_last


def ss_scan_fwd_static(u, delta, A, Bmat, Cmat, Dskip=None, z=None, delta_bias=None, h0=None,
                       delta_softplus=False, *, out, h_last=None, exact_zoh=False, complex_state=False, stream=None):
    """Enqueue the plain forward scan with the library's own static device scratch: the call
    allocates nothing, so ``out`` (and ``h_last`` if wanted) must be given.  Returns (out, h_last)."""
    import torch
    p = _fwd_params(u, delta, A, Bmat, Cmat, Dskip, z, delta_bias, h0, delta_softplus, exact_zoh, complex_state)
    state_shape = (p.batch, p.dim, p.dstate) + ((2,) if complex_state else ())
    p.out = _ptr(out, u.dtype, u.shape, "out")
    if h_last is not None:
        p.h_last = _ptr(h_last, torch.float32, state_shape, "h_last")
        p.flags |= SS_WRITE_H_LAST
    rc = lib().ss_scan_fwd_static(ctypes.byref(p), _stream(stream))
    if rc != SS_OK:
        raise SsError(rc)
    return out, h_last


def ss_scan_bwd(dout, u, delta, A, Bmat, Cmat, workspace, Dskip=None, z=None, delta_bias=None,
                h0=None, delta_softplus=False, dh_last=None, want_dh0=False, exact_zoh=False, complex_state=False,
                stream=None, grads=None):
    """Enqueue the backward scan after a forward call that filled ``workspace``.

    Returns a dict with du, ddelta, dz, dB, dC, dA, dD, ddelta_bias, dh0 (None where the
    corresponding input was not given).  ``grads``: a dict an earlier call returned; its
    tensors are written again instead of allocating new ones.  Freshly allocated du, ddelta and dz
    are views into one allocation (``empty_channel_skewed``): it lives as long as any of them."""
    import torch
    f32 = torch.float32
    q = BwdParams()
    q.fwd = _fwd_params(u, delta, A, Bmat, Cmat, Dskip, z, delta_bias, h0, delta_softplus, exact_zoh, complex_state)
    nb, nd, nl, nn = q.fwd.batch, q.fwd.dim, q.fwd.seqlen, q.fwd.dstate
    state_shape = (nb, nd, nn) + ((2,) if complex_state else ())
    q.fwd.workspace = _ptr(workspace, torch.uint8, None, "workspace")
    q.fwd.workspace_bytes = workspace.numel()
    dev = u.device
    fresh = empty_channel_skewed(3 if z is not None else 2, u.shape, u.dtype, dev) if grads is None else None
    g = grads if grads is not None else {
         "du": fresh[0], "ddelta": fresh[1],
         "dz": fresh[2] if z is not None else None,
         "dB": torch.empty(tuple(Bmat.shape), dtype=f32, device=dev),
         "dC": torch.empty(tuple(Cmat.shape), dtype=f32, device=dev),
         "dA": torch.empty(tuple(A.shape), dtype=f32, device=dev),
         "dD": torch.empty((nd,), dtype=f32, device=dev) if Dskip is not None else None,
         "ddelta_bias": torch.empty((nd,), dtype=f32, device=dev) if delta_bias is not None else None,
         "dh0": torch.empty(state_shape, dtype=f32, device=dev) if want_dh0 else None}
    if grads is not None:   # same checks as for fresh tensors: shapes and dtypes of what will be written
        want = {"du": (u.dtype, u.shape), "ddelta": (u.dtype, u.shape), "dz": (u.dtype, u.shape),
                "dB": (f32, Bmat.shape), "dC": (f32, Cmat.shape), "dA": (f32, A.shape), "dD": (f32, (nd,)),
                "ddelta_bias": (f32, (nd,)), "dh0": (f32, state_shape)}
        need = {"du": True, "ddelta": True, "dz": z is not None, "dB": True, "dC": True, "dA": True,
                "dD": Dskip is not None, "ddelta_bias": delta_bias is not None, "dh0": want_dh0}
        for name, (dt, shp) in want.items():
            if need[name] and grads.get(name) is None:
                raise ValueError("grads[%r] is missing" % name)
            if not need[name] and grads.get(name) is not None:
                raise ValueError("grads[%r] given but that gradient is not produced" % name)
            _ptr(grads.get(name), dt, shp, "grads[%r]" % name)
    q.dout = _ptr(dout, u.dtype, u.shape, "dout")
    q.dh_last = _ptr(dh_last, f32, state_shape, "dh_last")
    for name in ("du", "ddelta", "dz", "dB", "dC", "dA", "dD", "ddelta_bias", "dh0"):
        setattr(q, name, _ptr(g[name], None, None, name))
    rc = lib().ss_scan_bwd(ctypes.byref(q), _stream(stream))
    if rc != SS_OK:
        raise SsError(rc)
    return g


def ss_step(h, u_t, delta_t, A, B_t, C_t, Dskip=None, z_t=None, delta_bias=None,
            delta_softplus=False, out_t=None, exact_zoh=False, b_fixed=False, c_fixed=False, complex_state=False,
            stream=None):
    """Enqueue one recurrent step; ``h`` (B,D,N) float32 is updated in place.  Returns out_t.
    With ``b_fixed`` / ``c_fixed`` B_t / C_t is the time-invariant (D,N) float32 parameter."""
    import torch
    f32 = torch.float32
    nb, nd, nn = h.shape[:3]
    c2 = (2,) if complex_state else ()
    io = u_t.dtype
    p = StepParams()
    p.batch, p.dim, p.dstate = nb, nd, nn
    p.io_dtype = _io_code(u_t)
    flags = (SS_DELTA_SOFTPLUS if delta_softplus else 0) | (SS_EXACT_ZOH_B if exact_zoh else 0)
    flags |= (SS_B_FIXED if b_fixed else 0) | (SS_C_FIXED if c_fixed else 0) | (SS_COMPLEX_STATE if complex_state else 0)
    p.h = _ptr(h, f32, (nb, nd, nn) + c2, "h")
    p.u_t = _ptr(u_t, io, (nb, nd), "u_t")
    p.delta_t = _ptr(delta_t, io, (nb, nd), "delta_t")
    p.B_t = _ptr(B_t, f32, (nd, nn) + c2, "B_t") if b_fixed else _ptr(B_t, io, (nb, nn) + c2, "B_t")
    p.C_t = _ptr(C_t, f32, (nd, nn) + c2, "C_t") if c_fixed else _ptr(C_t, io, (nb, nn) + c2, "C_t")
    p.A = _ptr(A, f32, (nd, nn) + c2, "A")
    if z_t is not None:
        p.z_t = _ptr(z_t, io, (nb, nd), "z_t")
        flags |= SS_HAS_Z
    if Dskip is not None:
        p.Dskip = _ptr(Dskip, f32, (nd,), "Dskip")
        flags |= SS_HAS_D
    if delta_bias is not None:
        p.delta_bias = _ptr(delta_bias, f32, (nd,), "delta_bias")
        flags |= SS_HAS_DELTA_BIAS
    p.flags = flags
    if out_t is None:
        out_t = torch.empty_like(u_t)
    p.out_t = _ptr(out_t, io, (nb, nd), "out_t")
    rc = lib().ss_step(ctypes.byref(p), _stream(stream))
    if rc != SS_OK:
        raise SsError(rc)
    return out_t


# ---------------------------------------------------------------- short causal convolution
def _conv_params(x, w, bias, state_in, silu):
    import torch
    f32 = torch.float32
    nb, nd, nl = x.shape
    width = w.shape[1]
    p = ConvParams()
    p.batch, p.dim, p.seqlen, p.width = nb, nd, nl, width
    p.io_dtype = _io_code(x)
    flags = SS_CONV_SILU if silu else 0
    p.x = _ptr(x, None, (nb, nd, nl), "x")
    p.w = _ptr(w, f32, (nd, width), "w")
    if bias is not None:
        p.bias = _ptr(bias, f32, (nd,), "bias")
        flags |= SS_CONV_HAS_BIAS
    if state_in is not None:
        p.state_in = _ptr(state_in, x.dtype, (nb, nd, width - 1), "state_in")
        flags |= SS_CONV_HAS_STATE
    p.flags = flags
    return p


def ss_conv_fwd(x, w, bias=None, state_in=None, silu=True, out=None, return_state=False, stream=None):
    """Enqueue the causal convolution (+ SiLU).  Returns (out, state_out or None)."""
    import torch
    p = _conv_params(x, w, bias, state_in, silu)
    if out is None:
        out = torch.empty_like(x)
    p.out = _ptr(out, x.dtype, x.shape, "out")
    state_out = None
    if return_state:
        state_out = torch.empty((p.batch, p.dim, p.width - 1), dtype=x.dtype, device=x.device)
        p.state_out = _ptr(state_out, None, None, "state_out")
        p.flags |= SS_CONV_WRITE_STATE
    rc = lib().ss_conv_fwd(ctypes.byref(p), _stream(stream))
    if rc != SS_OK:
        raise SsError(rc)
    return out, state_out


def ss_conv_bwd(dout, x, w, bias=None, state_in=None, silu=True, stream=None):
    """Enqueue the backward convolution.  Returns dict(dx, dw, dbias)."""
    import torch
    q = ConvBwdParams()
    q.fwd = _conv_params(x, w, bias, state_in, silu)
    g = {"dx": torch.empty_like(x), "dw": torch.empty_like(w),
         "dbias": torch.empty_like(bias) if bias is not None else None}
    q.dout = _ptr(dout, x.dtype, x.shape, "dout")
    q.dx = _ptr(g["dx"], None, None, "dx")
    q.dw = _ptr(g["dw"], None, None, "dw")
    q.dbias = _ptr(g["dbias"], None, None, "dbias")
    rc = lib().ss_conv_bwd(ctypes.byref(q), _stream(stream))
    if rc != SS_OK:
        raise SsError(rc)
    return g


def ss_conv_step(state, x_t, w, bias=None, silu=True, out_t=None, stream=None):
    """Enqueue one token of the convolution; ``state`` (B,D,W-1) is updated in place."""
    import torch
    nb, nd = x_t.shape
    width = w.shape[1]
    p = ConvStepParams()
    p.batch, p.dim, p.width = nb, nd, width
    p.io_dtype = _io_code(x_t)
    p.flags = (SS_CONV_SILU if silu else 0) | (SS_CONV_HAS_BIAS if bias is not None else 0)
    p.state = _ptr(state, x_t.dtype, (nb, nd, width - 1), "state")
    p.x_t = _ptr(x_t, None, (nb, nd), "x_t")
    p.w = _ptr(w, torch.float32, (nd, width), "w")
    p.bias = _ptr(bias, torch.float32, (nd,), "bias")
    if out_t is None:
        out_t = torch.empty_like(x_t)
    p.out_t = _ptr(out_t, x_t.dtype, (nb, nd), "out_t")
    rc = lib().ss_conv_step(ctypes.byref(p), _stream(stream))
    if rc != SS_OK:
        raise SsError(rc)
    return out_t


# ---------------------------------------------------------------- the selective SSM layer
def _layer_shape(batch, dim, seqlen, dstate, dt_rank, conv_width, io_dtype):
    p = LayerParams()
    p.batch, p.dim, p.seqlen, p.dstate, p.dt_rank, p.conv_width = batch, dim, seqlen, dstate, dt_rank, conv_width
    p.io_dtype = io_dtype
    return p


def ss_layer_saved_bytes(batch, dim, seqlen, dstate, dt_rank, conv_width=4, io_dtype=SS_BF16):
    return int(lib().ss_layer_saved_bytes(ctypes.byref(
        _layer_shape(batch, dim, seqlen, dstate, dt_rank, conv_width, io_dtype))))


def ss_layer_scratch_bytes(batch, dim, seqlen, dstate, dt_rank, conv_width=4, io_dtype=SS_BF16, for_backward=True):
    return int(lib().ss_layer_scratch_bytes(ctypes.byref(
        _layer_shape(batch, dim, seqlen, dstate, dt_rank, conv_width, io_dtype)), int(bool(for_backward))))


def _layer_params(x, z, conv_w, conv_b, W_x, W_dt, dt_bias, A, Dskip, saved, scratch):
    import torch
    f32 = torch.float32
    nb, nd, nl = x.shape
    nn = A.shape[1]
    rank = W_dt.shape[1]
    width = conv_w.shape[1]
    io = x.dtype
    p = _layer_shape(nb, nd, nl, nn, rank, width, _io_code(x))
    p.x = _ptr(x, io, (nb, nd, nl), "x")
    p.z = _ptr(z, io, (nb, nd, nl), "z")
    p.conv_w = _ptr(conv_w, f32, (nd, width), "conv_w")
    p.conv_b = _ptr(conv_b, f32, (nd,), "conv_b")
    p.W_x = _ptr(W_x, io, (rank + 2 * nn, nd), "W_x")
    p.W_dt = _ptr(W_dt, io, (nd, rank), "W_dt")
    p.dt_bias = _ptr(dt_bias, f32, (nd,), "dt_bias")
    p.A = _ptr(A, f32, (nd, nn), "A")
    p.Dskip = _ptr(Dskip, f32, (nd,), "Dskip")
    if saved is not None:
        p.saved = _ptr(saved, torch.uint8, None, "saved")
        p.saved_bytes = saved.numel()
    p.scratch = _ptr(scratch, torch.uint8, None, "scratch")
    p.scratch_bytes = scratch.numel()
    return p


def ss_layer_fwd(x, z, conv_w, conv_b, W_x, W_dt, dt_bias, A, Dskip, scratch, saved=None, out=None,
                 return_states=False, stream=None, h_last=None, conv_state=None):
    """Enqueue the layer's forward pass; ``saved`` (if given) is filled for ``ss_layer_bwd``.
    Returns out, or (out, h_last, conv_state) with ``return_states`` (written into the caller's
    ``h_last`` (B,D,N) float32 and ``conv_state`` (B,D,W-1) tensors if given)."""
    import torch
    p = _layer_params(x, z, conv_w, conv_b, W_x, W_dt, dt_bias, A, Dskip, saved, scratch)
    if out is None:
        out = torch.empty_like(x)
    p.out = _ptr(out, x.dtype, x.shape, "out")
    if return_states:
        if h_last is None:
            h_last = torch.empty((p.batch, p.dim, p.dstate), dtype=torch.float32, device=x.device)
        if conv_state is None:
            conv_state = torch.empty((p.batch, p.dim, p.conv_width - 1), dtype=x.dtype, device=x.device)
        p.h_last = _ptr(h_last, torch.float32, (p.batch, p.dim, p.dstate), "h_last")
        p.conv_state = _ptr(conv_state, x.dtype, (p.batch, p.dim, p.conv_width - 1), "conv_state")
    rc = lib().ss_layer_fwd(ctypes.byref(p), _stream(stream))
    if rc != SS_OK:
        raise SsError(rc)
    return (out, h_last, conv_state) if return_states else out


def ss_layer_step_scratch_bytes(batch, dim, dstate, dt_rank, io_dtype=SS_BF16):
    p = LayerStepParams()
    p.batch, p.dim, p.dstate, p.dt_rank, p.conv_width, p.io_dtype = batch, dim, dstate, dt_rank, 4, io_dtype
    return int(lib().ss_layer_step_scratch_bytes(ctypes.byref(p)))


def ss_layer_step(h, conv_state, x_t, z_t, conv_w, conv_b, W_x, W_dt, dt_bias, A, Dskip, scratch, out_t=None,
                  stream=None):
    """Enqueue one token of the layer; ``h`` (B,D,N) and ``conv_state`` (B,D,W-1) are updated in place."""
    import torch
    f32 = torch.float32
    nb, nd, nn = h.shape
    rank = W_dt.shape[1]
    width = conv_w.shape[1]
    io = x_t.dtype
    p = LayerStepParams()
    p.batch, p.dim, p.dstate, p.dt_rank, p.conv_width = nb, nd, nn, rank, width
    p.io_dtype = _io_code(x_t)
    p.h = _ptr(h, f32, (nb, nd, nn), "h")
    p.conv_state = _ptr(conv_state, io, (nb, nd, width - 1), "conv_state")
    p.x_t = _ptr(x_t, io, (nb, nd), "x_t")
    p.z_t = _ptr(z_t, io, (nb, nd), "z_t")
    p.conv_w = _ptr(conv_w, f32, (nd, width), "conv_w")
    p.conv_b = _ptr(conv_b, f32, (nd,), "conv_b")
    p.W_x = _ptr(W_x, io, (rank + 2 * nn, nd), "W_x")
    p.W_dt = _ptr(W_dt, io, (nd, rank), "W_dt")
    p.dt_bias = _ptr(dt_bias, f32, (nd,), "dt_bias")
    p.A = _ptr(A, f32, (nd, nn), "A")
    p.Dskip = _ptr(Dskip, f32, (nd,), "Dskip")
    if out_t is None:
        out_t = torch.empty_like(x_t)
    p.out_t = _ptr(out_t, io, (nb, nd), "out_t")
    p.scratch = _ptr(scratch, torch.uint8, None, "scratch")
    p.scratch_bytes = scratch.numel()
    rc = lib().ss_layer_step(ctypes.byref(p), _stream(stream))
    if rc != SS_OK:
        raise SsError(rc)
    return out_t


def ss_layer_bwd(dout, x, z, conv_w, conv_b, W_x, W_dt, dt_bias, A, Dskip, scratch, saved, stream=None):
    """Enqueue the layer's backward pass.  Returns a dict of gradients (weights in float32)."""
    import torch
    f32 = torch.float32
    q = LayerBwdParams()
    q.fwd = _layer_params(x, z, conv_w, conv_b, W_x, W_dt, dt_bias, A, Dskip, saved, scratch)
    dev = x.device
    g = {"dx": torch.empty_like(x), "dz": torch.empty_like(x),
         "dconv_w": torch.empty_like(conv_w), "dconv_b": torch.empty_like(conv_b),
         "dW_x": torch.empty(W_x.shape, dtype=f32, device=dev), "dW_dt": torch.empty(W_dt.shape, dtype=f32, device=dev),
         "ddt_bias": torch.empty_like(dt_bias), "dA": torch.empty_like(A), "dD": torch.empty_like(Dskip)}
    q.dout = _ptr(dout, x.dtype, x.shape, "dout")
    for name, t in g.items():
        setattr(q, name, _ptr(t, None, None, name))
    rc = lib().ss_layer_bwd(ctypes.byref(q), _stream(stream))
    if rc != SS_OK:
        raise SsError(rc)
    return g


def ss_proj_gemm(A, B, C, trans_a=False, trans_b=False, accumulate=False, general=False, stream=None, workspace=None):
    """C[i] = op(A[i]) @ op(B[i]) (+ C[i]) on the layer's projection kernels.  A, B, C are 2-D or
    3-D (leading batch axis) tensors whose last axis is contiguous; a 2-D operand is shared by all
    batch entries.  ``trans_a`` / ``trans_b``: the operand is stored transposed ((K, M) / (N, K)).
    C is float32 or of the operands' dtype.  ``workspace``: optional uint8 device tensor of
    ``ss_proj_gemm_workspace_bytes(C)`` bytes that lets a product with few rows and columns split its
    contraction across workgroups."""
    import torch
    def view(t):
        if t.stride(-1) != 1:
            raise ValueError("the last axis must be contiguous")
        return (t.shape[0], t.stride(0), t.stride(1)) if t.dim() == 3 else (1, 0, t.stride(0))
    (ba, sa, lda), (bb, sb, ldb), (bc, sc, ldc) = view(A), view(B), view(C)
    if C.dim() == 3 and C.shape[0] > 1 and sc == 0:
        raise ValueError("C needs its own batch entries")
    p = GemmParams()
    p.M, p.N = C.shape[-2], C.shape[-1]
    p.K = A.shape[-2] if trans_a else A.shape[-1]
    kb = B.shape[-1] if trans_b else B.shape[-2]
    ma = A.shape[-1] if trans_a else A.shape[-2]
    nb_ = B.shape[-2] if trans_b else B.shape[-1]
    if kb != p.K or ma != p.M or nb_ != p.N or A.dtype != B.dtype:
        raise ValueError("shapes or dtypes do not agree")
    p.batch = bc if C.dim() == 3 else 1
    for t, n in ((A, ba), (B, bb)):
        if t.dim() == 3 and n != p.batch:
            raise ValueError("batch sizes do not agree")
    p.io_dtype = _io_code(A)
    if C.dtype == torch.float32:
        p.flags |= SS_GEMM_C_FLOAT
    elif C.dtype != A.dtype:
        raise ValueError("C must be float32 or of the operands' dtype")
    if accumulate:
        p.flags |= SS_GEMM_ACCUMULATE
    if general:
        p.flags |= SS_GEMM_GENERAL
    p.A, p.B, p.C = A.data_ptr(), B.data_ptr(), C.data_ptr()
    p.a_m, p.a_k = (1, lda) if trans_a else (lda, 1)
    p.b_k, p.b_n = (1, ldb) if trans_b else (ldb, 1)
    p.a_batch, p.b_batch, p.ldc, p.c_batch = sa, sb, ldc, sc
    for t in (A, B, C):
        if not t.is_cuda:
            raise ValueError("device tensors expected")
    if workspace is not None:
        if not workspace.is_cuda:
            raise ValueError("device tensors expected")
        p.workspace, p.workspace_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    rc = lib().ss_proj_gemm(ctypes.byref(p), _stream(stream))
    if rc != SS_OK:
        raise SsError(rc)
    return C


def ss_proj_gemm_workspace_bytes(C):
    """Bytes of workspace with which ``ss_proj_gemm`` may split the contraction of a product with result ``C``."""
    p = GemmParams()
    p.M, p.N = C.shape[-2], C.shape[-1]
    p.batch = C.shape[0] if C.dim() == 3 else 1
    return int(lib().ss_proj_gemm_workspace_bytes(ctypes.byref(p)))
