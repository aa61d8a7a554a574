"""Float64 CPU oracle of the selective SSM layer: conv -> SiLU -> projections -> scan -> gate.

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the benchmark's
``cpu_baseline`` leg import this module; the product path never does.

This is Algorithm 2 of the paper with the selection functions of Section 3.2 and the
low-rank Delta of Section 3.6, preceded by the short convolution and SiLU of the block in
Section 3.4 (Figure 3) and followed by its multiplicative gate.  With the sequence axis
last, for every batch entry b:

    u          = SiLU(conv(x))                         (D, L)    conv_oracle.conv_fwd
    [r; B; C]  = W_x @ u                               (R+N+N, L)   s_Delta (rank R), s_B, s_C
    delta_raw  = W_dt @ r                              (D, L)    Linear_D after Linear_R
    out        = scan(u, softplus(delta_raw + dt_bias), A, B, C, D) * SiLU(z)

Each step is the definition, composed from the conv and scan oracles and numpy matmul.
``rnd`` (identity by default) is applied to u, [r;B;C] and delta_raw: the layer's
interface stores those three intermediates in the io dtype, so a bf16 run rounds them and
the oracle must round at the same three places to describe the same function.  In the
backward pass ``rnd`` is treated as the identity map (gradients pass straight through).
"""
import numpy as np

from . import conv_oracle, ss_oracle


def _f64(a):
    return None if a is None else np.asarray(a, dtype=np.float64)


def _identity(a):
    return a


def inner_fwd(x, z, conv_w, conv_b, W_x, W_dt, dt_bias, A, Dskip, rnd=None, nthreads=0):
    """Returns dict(out, u, P, delta_raw, h_last, conv_state); P = [r; B; C] stacked along axis 1.
    h_last (B,D,N) and conv_state (B,D,W-1) are what the recurrent mode continues from."""
    rnd = rnd or _identity
    x, W_x, W_dt = _f64(x), _f64(W_x), _f64(W_dt)
    N = np.asarray(A).shape[1]
    R = W_dt.shape[1]
    assert W_x.shape == (R + 2 * N, x.shape[1])
    c = conv_oracle.conv_fwd(x, conv_w, conv_b, None, silu=True)
    u = rnd(c["out"])
    P = rnd(np.matmul(W_x[None], u))                       # (B, R+2N, L)
    delta_raw = rnd(np.matmul(W_dt[None], P[:, :R]))       # (B, D, L)
    s = ss_oracle.scan_fwd(u, delta_raw, A, P[:, R:R + N], P[:, R + N:], Dskip=Dskip, z=z,
                           bias=dt_bias, softplus=True, nthreads=nthreads)
    return {"out": s["out"], "u": u, "P": P, "delta_raw": delta_raw, "h_last": s["h_last"],
            "conv_state": c["state_out"]}


def inner_step(h, conv_state, x_t, z_t, conv_w, conv_b, W_x, W_dt, dt_bias, A, Dskip, rnd=None):
    """One token of the layer in recurrent mode (Section 2; Eq. 2a/2b applied once after the
    sliding conv window).  h (B,D,N), conv_state (B,D,W-1), x_t, z_t (B,D).
    Returns (out_t (B,D), new h, new conv_state); the inputs are not modified."""
    rnd = rnd or _identity
    W_x, W_dt = _f64(W_x), _f64(W_dt)
    N = np.asarray(A).shape[1]
    R = W_dt.shape[1]
    u_t, conv_state = conv_oracle.conv_step(conv_state, x_t, conv_w, conv_b, silu=True)
    u_t = rnd(u_t)
    P_t = rnd(u_t @ W_x.T)                                 # (B, R+2N)
    delta_t = rnd(P_t[:, :R] @ W_dt.T)                     # (B, D)
    out_t, h = ss_oracle.step(h, u_t, delta_t, A, P_t[:, R:R + N], P_t[:, R + N:], Dskip=Dskip, z_t=z_t,
                              bias=dt_bias, softplus=True)
    return out_t, h, conv_state


def inner_bwd(x, z, conv_w, conv_b, W_x, W_dt, dt_bias, A, Dskip, dout, rnd=None, nthreads=0):
    """Gradient of <out, dout> w.r.t. every input of inner_fwd."""
    x, W_x, W_dt = _f64(x), _f64(W_x), _f64(W_dt)
    N = np.asarray(A).shape[1]
    R = W_dt.shape[1]
    f = inner_fwd(x, z, conv_w, conv_b, W_x, W_dt, dt_bias, A, Dskip, rnd, nthreads)
    u, P = f["u"], f["P"]
    g = ss_oracle.scan_bwd(u, f["delta_raw"], A, P[:, R:R + N], P[:, R + N:], dout, Dskip=Dskip, z=z,
                           bias=dt_bias, softplus=True, nthreads=nthreads)
    # delta_raw = W_dt @ r
    dW_dt = np.einsum("bdl,brl->dr", g["ddelta"], P[:, :R])
    dr = np.matmul(W_dt.T[None], g["ddelta"])              # (B, R, L)
    # [r; B; C] = W_x @ u
    dP = np.concatenate([dr, g["dB"], g["dC"]], axis=1)
    dW_x = np.einsum("bml,bdl->md", dP, u)
    du = g["du"] + np.matmul(W_x.T[None], dP)
    c = conv_oracle.conv_bwd(x, conv_w, du, conv_b, None, silu=True)
    return {"dx": c["dx"], "dz": g["dz"], "dconv_w": c["dw"], "dconv_b": c["dbias"], "dW_x": dW_x,
            "dW_dt": dW_dt, "ddt_bias": g["dbias"], "dA": g["dA"], "dD": g["dD"]}
