"""Float64 / complex128 CPU oracle of the selective scan with a complex-valued state.

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the benchmark's
``cpu_baseline`` leg import this module; the product path never does.

The paper keeps the state real by default and switches to a complex state for one experiment
(Section 3.6 "Real vs. Complex"; S4D-Lin initialisation A_n = -1/2 + n i); it does not spell
the complex case out.  This oracle takes Eq. 2a/2b/4 over the complex numbers as they stand,
with the real part as the output (a reading: the paper does not say how y becomes real):

    abar_t,n = exp(dt_t * A[d,n])                       A, abar complex        (Eq. 4)
    h_t,n    = abar_t,n * h_{t-1,n} + dt_t * B[b,n,t] * u[b,d,t]   B, h complex (Eq. 2a, first-order B-bar)
    y_t      = Re( sum_n C[b,n,t] * h_t,n ) + Dskip[d] * u[b,d,t]  C complex    (Eq. 2b)
    out_t    = y_t * z_t * sigmoid(z_t)

dt = softplus(delta + bias) as in the real case; u, delta, z, out are real.  The functions are
the definition, one time step after the other, vectorised only over (b, d, n).
Layouts: u, delta, z (B,D,L) real; A (D,N) complex; B, C (B,N,L) complex; h0 (B,D,N) complex.
The gradient of a real loss w.r.t. a complex input p is returned as dL/dRe(p) + i dL/dIm(p).
"""
import numpy as np


def _softplus(r):
    return np.maximum(r, 0.0) + np.log1p(np.exp(-np.abs(r)))


def _sigmoid(v):
    return 1.0 / (1.0 + np.exp(-v))


def _prep(u, delta, A, Bm, Cm, Dskip, z, bias, h0, softplus):
    u = np.asarray(u, np.float64)
    delta = np.asarray(delta, np.float64)
    A = np.asarray(A, np.complex128)
    Bm = np.asarray(Bm, np.complex128)
    Cm = np.asarray(Cm, np.complex128)
    nb, nd, nl = u.shape
    nn = A.shape[1]
    assert A.shape == (nd, nn) and Bm.shape == (nb, nn, nl) and Cm.shape == (nb, nn, nl)
    r = delta + (0.0 if bias is None else np.asarray(bias, np.float64)[None, :, None])
    dt = _softplus(r) if softplus else r
    h = np.zeros((nb, nd, nn), np.complex128) if h0 is None else np.array(h0, np.complex128)
    return u, A, Bm, Cm, r, dt, h


def scan_fwd(u, delta, A, Bm, Cm, Dskip=None, z=None, bias=None, h0=None, softplus=False):
    """Returns dict(out (B,D,L) real, h_last (B,D,N) complex, y_pre)."""
    u, A, Bm, Cm, r, dt, h = _prep(u, delta, A, Bm, Cm, Dskip, z, bias, h0, softplus)
    nb, nd, nl = u.shape
    y = np.empty((nb, nd, nl))
    for t in range(nl):
        abar = np.exp(dt[:, :, t, None] * A[None])                           # (B,D,N)
        h = abar * h + dt[:, :, t, None] * Bm[:, None, :, t] * u[:, :, t, None]
        y[:, :, t] = np.real(np.sum(Cm[:, None, :, t] * h, axis=2))
    if Dskip is not None:
        y = y + np.asarray(Dskip, np.float64)[None, :, None] * u
    out = y if z is None else y * np.asarray(z, np.float64) * _sigmoid(np.asarray(z, np.float64))
    return {"out": out, "h_last": h, "y_pre": y}


def scan_bwd(u, delta, A, Bm, Cm, dout, Dskip=None, z=None, bias=None, h0=None, dh_last=None, softplus=False):
    """Gradient of <out, dout> + Re<h_last, conj(dh_last)> (i.e. the sum over real and imaginary
    parts of h_last times those of dh_last) w.r.t. every input.  Complex gradients are
    dL/dRe + i dL/dIm.  Returns dict(du, ddelta, dz, dB, dC, dA, dD, dbias, dh0)."""
    u, A, Bm, Cm, r, dt, h = _prep(u, delta, A, Bm, Cm, Dskip, z, bias, h0, softplus)
    dout = np.asarray(dout, np.float64)
    nb, nd, nl = u.shape
    nn = A.shape[1]
    # every state, stored: hs[t] = h_t, hs[-1 + 0] handled through h_init
    h_init = h
    hs = np.empty((nl, nb, nd, nn), np.complex128)
    for t in range(nl):
        abar = np.exp(dt[:, :, t, None] * A[None])
        h = abar * h + dt[:, :, t, None] * Bm[:, None, :, t] * u[:, :, t, None]
        hs[t] = h
    y = np.empty((nb, nd, nl))
    for t in range(nl):
        y[:, :, t] = np.real(np.sum(Cm[:, None, :, t] * hs[t], axis=2))
    if Dskip is not None:
        y = y + np.asarray(Dskip, np.float64)[None, :, None] * u
    if z is not None:
        zz = np.asarray(z, np.float64)
        s = _sigmoid(zz)
        dz = dout * y * s * (1.0 + zz * (1.0 - s))
        dy = dout * zz * s
    else:
        dz = None
        dy = dout
    du = np.zeros_like(u)
    ddt = np.zeros_like(u)
    dA = np.zeros((nd, nn), np.complex128)
    dB = np.zeros((nb, nn, nl), np.complex128)
    dC = np.zeros((nb, nn, nl), np.complex128)
    dD = None
    if Dskip is not None:
        du += np.asarray(Dskip, np.float64)[None, :, None] * dy
        dD = np.sum(dy * u, axis=(0, 2))
    # g = dL/dRe(h) + i dL/dIm(h).  For w = a * v (complex product) and a real loss,
    # grad_v = conj(a) * grad_w and grad_a = conj(v) * grad_w in this convention.
    g = np.zeros((nb, nd, nn), np.complex128) if dh_last is None else np.array(dh_last, np.complex128)
    for t in range(nl - 1, -1, -1):
        dtt = dt[:, :, t, None]
        ut = u[:, :, t, None]
        abar = np.exp(dtt * A[None])
        hprev = hs[t - 1] if t > 0 else h_init
        Ct = Cm[:, None, :, t]
        Bt = Bm[:, None, :, t]
        # y_t = Re(sum C h_t):  grad_h += conj(C) dy,  grad_C = conj(h) dy
        g = g + np.conj(Ct) * dy[:, :, t, None]
        dC[:, :, t] = np.sum(np.conj(hs[t]) * dy[:, :, t, None], axis=1)
        # h_t = abar hprev + dt B u
        g_abar = np.conj(hprev) * g                     # gradient w.r.t. abar
        g_b = g                                          # gradient w.r.t. the input term dt*B*u
        dB[:, :, t] = np.sum(g_b * dtt * ut, axis=1)     # conj(dt u) = dt u (real)
        du[:, :, t] += np.sum(np.real(np.conj(dtt * Bt) * g_b), axis=2)
        # abar = exp(dt A): grad_A = conj(dt abar) g_abar, and dt is real: d/ddt = Re(conj(A abar) g_abar)
        dA += np.sum(np.conj(dtt * abar) * g_abar, axis=0)
        ddt[:, :, t] = np.sum(np.real(np.conj(A[None] * abar) * g_abar) + np.real(np.conj(Bt * ut) * g_b), axis=2)
        g = np.conj(abar) * g                            # flows on to h_{t-1}
    ddelta = ddt * _sigmoid(r) if softplus else ddt
    dbias = None if bias is None else np.sum(ddelta, axis=(0, 2))
    return {"du": du, "ddelta": ddelta, "dz": dz, "dB": dB, "dC": dC, "dA": dA, "dD": dD, "dbias": dbias, "dh0": g}


def step(h, u_t, delta_t, A, B_t, C_t, Dskip=None, z_t=None, bias=None, softplus=False):
    """One recurrent step.  h (B,D,N) complex, B_t, C_t (B,N) complex.  Returns (out_t, new h)."""
    h = np.array(h, np.complex128)
    u_t = np.asarray(u_t, np.float64)
    A = np.asarray(A, np.complex128)
    r = np.asarray(delta_t, np.float64) + (0.0 if bias is None else np.asarray(bias, np.float64)[None, :])
    dt = _softplus(r) if softplus else r
    abar = np.exp(dt[:, :, None] * A[None])
    h = abar * h + dt[:, :, None] * np.asarray(B_t, np.complex128)[:, None, :] * u_t[:, :, None]
    y = np.real(np.sum(np.asarray(C_t, np.complex128)[:, None, :] * h, axis=2))
    if Dskip is not None:
        y = y + np.asarray(Dskip, np.float64)[None, :] * u_t
    if z_t is not None:
        zz = np.asarray(z_t, np.float64)
        y = y * zz * _sigmoid(zz)
    return y, h
