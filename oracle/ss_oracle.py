"""ctypes front-end of the float64 CPU oracle in ``ss_oracle.c``.

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the benchmark's
``cpu_baseline`` leg import this module; the product path never does.  It shares
nothing with the HIP library (no headers, constants or helpers).

Every function takes numpy arrays of any float dtype (they are widened to
contiguous float64) in the layouts of the paper's Algorithm 2 with the sequence
axis last: u/delta/z (B,D,L), B/C (B,N,L), A (D,N), Dskip/bias (D), h0 (B,D,N).
B or C given as a 2-D (D,N) array is taken as time-invariant (Algorithm 1; the
non-selective arms of the ablation in Table 7); its gradient then has that shape too.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ss_oracle.c")
_LIB = os.path.join(_HERE, "libss_oracle.so")
_lib = None


def build(force=False):
    """Compile ss_oracle.c with gcc into libss_oracle.so next to it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
               "-ffp-contract=off", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.c_void_p
        i = ctypes.c_int
        lib.ss_oracle_fwd.restype = i
        lib.ss_oracle_fwd.argtypes = [i, i, ctypes.c_long, i] + [dp] * 9 + [i, i, i, i] + [dp] * 3 + [i]
        lib.ss_oracle_bwd.restype = i
        lib.ss_oracle_bwd.argtypes = ([i, i, ctypes.c_long, i] + [dp] * 9 + [i, i, i, i]
                                      + [dp] * 2 + [dp] * 9 + [i])
        lib.ss_oracle_step.restype = i
        lib.ss_oracle_step.argtypes = [i, i, i] + [dp] * 9 + [i, i, i, i] + [dp]
        lib.ss_oracle_threads.restype = i
        _lib = lib
    return _lib


def threads():
    """Number of host threads the oracle uses by default."""
    return int(_load().ss_oracle_threads())


def _f64(a):
    return None if a is None else np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _fixed(M, nb, nd, nl, nn, name):
    """True if M is the time-invariant (D,N) form (Algorithm 1), False for the selective (B,N,L)."""
    if M.ndim == 2:
        assert M.shape == (nd, nn), "%s must be (D,N) when time-invariant" % name
        return True
    assert M.shape == (nb, nn, nl), "%s must be (B,N,L)" % name
    return False


def _shapes(u, Bm, Cm, A):
    nb, nd, nl = u.shape
    nn = A.shape[1]
    assert A.shape == (nd, nn), "A must be (D,N)"
    return nb, nd, nl, nn, _fixed(Bm, nb, nd, nl, nn, "B"), _fixed(Cm, nb, nd, nl, nn, "C")


def scan_fwd(u, delta, A, Bm, Cm, Dskip=None, z=None, bias=None, h0=None,
             softplus=False, exact_zoh=False, nthreads=0):
    """Selective scan forward.  Returns dict(out, h_last, y_pre) of float64 arrays."""
    u, delta, A, Bm, Cm = map(_f64, (u, delta, A, Bm, Cm))
    Dskip, z, bias, h0 = map(_f64, (Dskip, z, bias, h0))
    nb, nd, nl, nn, bfix, cfix = _shapes(u, Bm, Cm, A)
    assert delta.shape == u.shape
    out = np.empty_like(u)
    y_pre = np.empty_like(u)
    h_last = np.empty((nb, nd, nn))
    rc = _load().ss_oracle_fwd(nb, nd, nl, nn, _ptr(u), _ptr(delta), _ptr(z), _ptr(Bm),
                               _ptr(Cm), _ptr(A), _ptr(Dskip), _ptr(bias), _ptr(h0),
                               int(softplus), int(exact_zoh), int(bfix), int(cfix), _ptr(out),
                               _ptr(h_last), _ptr(y_pre), int(nthreads))
    if rc != 0:
        raise RuntimeError("ss_oracle_fwd failed: %d" % rc)
    return {"out": out, "h_last": h_last, "y_pre": y_pre}


def scan_bwd(u, delta, A, Bm, Cm, dout, Dskip=None, z=None, bias=None, h0=None,
             dh_last=None, softplus=False, exact_zoh=False, nthreads=0):
    """Gradient of <out,dout> + <h_last,dh_last> w.r.t. every input.

    Returns dict(du, ddelta, dz, dB, dC, dA, dD, dbias, dh0); entries whose input
    was not given are None."""
    u, delta, A, Bm, Cm, dout = map(_f64, (u, delta, A, Bm, Cm, dout))
    Dskip, z, bias, h0, dh_last = map(_f64, (Dskip, z, bias, h0, dh_last))
    nb, nd, nl, nn, bfix, cfix = _shapes(u, Bm, Cm, A)
    du = np.empty_like(u)
    ddelta = np.empty_like(u)
    dz = np.empty_like(u) if z is not None else None
    dB = np.empty_like(Bm)
    dC = np.empty_like(Cm)
    dA = np.empty_like(A)
    dD = np.empty(nd) if Dskip is not None else None
    dbias = np.empty(nd) if bias is not None else None
    dh0 = np.empty((nb, nd, nn))
    rc = _load().ss_oracle_bwd(nb, nd, nl, nn, _ptr(u), _ptr(delta), _ptr(z), _ptr(Bm),
                               _ptr(Cm), _ptr(A), _ptr(Dskip), _ptr(bias), _ptr(h0),
                               int(softplus), int(exact_zoh), int(bfix), int(cfix), _ptr(dout), _ptr(dh_last),
                               _ptr(du), _ptr(ddelta), _ptr(dz), _ptr(dB), _ptr(dC),
                               _ptr(dA), _ptr(dD), _ptr(dbias), _ptr(dh0), int(nthreads))
    if rc != 0:
        raise RuntimeError("ss_oracle_bwd failed: %d" % rc)
    return {"du": du, "ddelta": ddelta, "dz": dz, "dB": dB, "dC": dC, "dA": dA,
            "dD": dD, "dbias": dbias, "dh0": dh0}


def step(h, u_t, delta_t, A, B_t, C_t, Dskip=None, z_t=None, bias=None,
         softplus=False, exact_zoh=False, b_fixed=None, c_fixed=None):
    """One recurrent step.  Returns (out_t (B,D), new h (B,D,N)); h is not modified."""
    h = np.array(h, dtype=np.float64, order="C", copy=True)
    u_t, delta_t, A, B_t, C_t = map(_f64, (u_t, delta_t, A, B_t, C_t))
    Dskip, z_t, bias = map(_f64, (Dskip, z_t, bias))
    nb, nd, nn = h.shape
    assert u_t.shape == (nb, nd) and A.shape == (nd, nn)
    # (B,N) per token, or the time-invariant (D,N); ambiguous only when B == D, where the caller's
    # b_fixed / c_fixed decide
    bfix = b_fixed if b_fixed is not None else (B_t.shape == (nd, nn) and nb != nd)
    cfix = c_fixed if c_fixed is not None else (C_t.shape == (nd, nn) and nb != nd)
    assert B_t.shape == ((nd, nn) if bfix else (nb, nn)) and C_t.shape == ((nd, nn) if cfix else (nb, nn))
    out = np.empty((nb, nd))
    rc = _load().ss_oracle_step(nb, nd, nn, _ptr(h), _ptr(u_t), _ptr(delta_t), _ptr(z_t),
                                _ptr(B_t), _ptr(C_t), _ptr(A), _ptr(Dskip), _ptr(bias),
                                int(softplus), int(exact_zoh), int(bfix), int(cfix), _ptr(out))
    if rc != 0:
        raise RuntimeError("ss_oracle_step failed: %d" % rc)
    return out, h
