"""The two float32 formulas the exact zero-order-hold kernels use (Eq. 4: B-bar = phi B with
phi = (exp(dt A) - 1)/A), evaluated here in numpy float32 exactly as the kernels write them and held
against the float64 closed forms.  This pins the error bounds the kernels' comments state and the
place where the small-argument series takes over; it needs no GPU and no oracle code.

  phi            = dt (1 + x/2 + x^2/6)              for |x| < 2^-7, x = dt A   (covers A = 0)
                 = (abar - 1) (1/A)                   otherwise, abar = exp(x) in float32
  g dphi/dA      = g dt^2 (1/2 + x/3 + x^2/8)         for |x| < 2^-4
                 = (abar g dt - g phi) (1/A)          otherwise (the difference magnifies phi's error by 2/|x|)
"""
import numpy as np

F = np.float32
LOG2E = F(1.4426950408889634)
LN2 = F(0.6931471805599453)
SMALL_X2 = F(0.0078125) * LOG2E
SMALL_X2_GRAD = F(0.0625) * LOG2E


def _grid():
    dt = np.exp(np.linspace(np.log(1e-9), np.log(30.0), 400)).astype(F)
    A = np.concatenate([-np.exp(np.linspace(np.log(1e-4), np.log(50.0), 120)), [0.0],
                        np.exp(np.linspace(np.log(1e-4), np.log(2.0), 30))]).astype(F)
    dt, A = np.meshgrid(dt, A)
    keep = dt.astype(np.float64) * A < 60.0          # keep exp in float32 range
    return dt[keep], A[keep]


def _kernel_terms(dt, A):
    A2 = A * LOG2E
    inv_A = np.where(A == 0, F(0), F(1) / np.where(A == 0, F(1), A)).astype(F)
    x2 = dt * A2
    abar = np.exp2(x2).astype(F)
    small = np.abs(x2) < SMALL_X2
    series = dt * (x2 * (x2 * (LN2 * LN2 / F(6)) + LN2 / F(2)) + F(1))
    phi = np.where(small, series, (abar - F(1)) * inv_A).astype(F)
    return x2, abar, inv_A, small, phi


def test_phi_matches_the_divided_difference():
    dt, A = _grid()
    _, _, _, small, phi = _kernel_terms(dt, A)
    d64, a64 = dt.astype(np.float64), A.astype(np.float64)
    x = d64 * a64
    ref = np.where(a64 == 0, d64, np.expm1(x) / np.where(a64 == 0, 1.0, a64))
    rel = np.abs(phi - ref) / np.abs(ref)
    assert small.any() and (~small).any()
    assert rel[small].max() < 2e-7           # the series, three terms, plus float32 rounding
    assert rel[~small].max() < 3e-5          # one ulp of the exponential over |x| >= 2^-7
    # and the decay factor the adjoint sweep rebuilds from phi: abar = 1 + phi A
    abar2 = (phi * A + F(1)).astype(F)
    # (a float32 exponential of a large argument carries the argument's rounding: |x| ulps)
    assert (np.abs(abar2 - np.exp(x)) / (np.maximum(1.0, np.exp(x)) * (1.0 + np.abs(x)))).max() < 2e-7


def test_gradient_term_without_dphi_dA():
    dt, A = _grid()
    x2, _, inv_A, _, phi = _kernel_terms(dt, A)
    small = np.abs(x2) < SMALL_X2_GRAD
    g = F(0.75)
    abar = (phi * A + F(1)).astype(F)
    ag = abar * g
    gphi = g * phi
    direct = (ag * dt - gphi) * inv_A
    series = (g * (dt * dt)) * (x2 * (x2 * (LN2 * LN2 / F(8)) + LN2 / F(3)) + F(0.5))
    got = np.where(small, series, direct).astype(np.float64)
    d64, a64 = dt.astype(np.float64), A.astype(np.float64)
    x = d64 * a64
    safe = np.where(np.abs(x) < 1e-5, 1.0, x)
    r = np.where(np.abs(x) < 1e-5, 0.5 + x / 3.0, (safe * np.exp(safe) - np.expm1(safe)) / (safe * safe))   # dphi/dA / dt^2
    ref = 0.75 * d64 * d64 * r
    # what matters is the error against the other term of dA_n, g abar h_prev dt with h_prev of the
    # order of phi (the state a unit input leaves): the term itself may cancel, its error may not grow
    scale = np.abs(ref) + 0.75 * np.exp(x) * d64 * np.abs(phi.astype(np.float64))
    err = np.abs(got - ref) / scale
    assert small.any() and (~small).any()
    assert err[small].max() < 2e-5           # three series terms: x^3/30 relative to 1/2 at |x| = 2^-4
    assert err[~small].max() < 5e-5          # phi's error (one ulp of the exponential over |x|) times 2/|x|, |x| >= 2^-4
