"""Float64 CPU oracle of the short causal convolution + SiLU in front of the selective SSM.

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the benchmark's
``cpu_baseline`` leg import this module; the product path never does.  It shares
nothing with the HIP library.

The paper's block (Section 3.4, Figure 3) puts a short per-channel convolution and the
SiLU activation between the input projection and the SSM; it gives neither the width nor
the indexing, so this oracle fixes them as follows (the usual left-padded, per-channel
cross-correlation of deep-learning libraries):

    v[b,d,t] = bias[d] + sum_{k=0}^{W-1} w[d,k] * x[b,d,t-(W-1)+k]
    out      = v * sigmoid(v)   (SiLU, Section 3.4)   or   v

where x at negative times is 0, or the W-1 samples ``state_in[b,d,:]`` that preceded the
sequence (oldest first).  ``state_out`` holds the last W-1 samples seen, which makes a
sequence processed in pieces, or one token at a time (Section 2, recurrent mode), equal to
the sequence processed whole.  Everything is written as the definition, one tap at a time.
"""
import numpy as np


def _f64(a):
    return None if a is None else np.asarray(a, dtype=np.float64)


def _history(x, width, state_in):
    """(B,D,W-1+L): the sequence with the W-1 samples that precede it in front."""
    Bsz, D, _ = x.shape
    if state_in is None:
        pre = np.zeros((Bsz, D, width - 1))
    else:
        pre = _f64(state_in)
        assert pre.shape == (Bsz, D, width - 1)
    return np.concatenate([pre, x], axis=2)


def sigmoid(v):
    return 1.0 / (1.0 + np.exp(-v))


def conv_fwd(x, w, bias=None, state_in=None, silu=True):
    """Returns dict(out, pre, state_out); pre is the convolution before the activation."""
    x, w, bias = _f64(x), _f64(w), _f64(bias)
    Bsz, D, L = x.shape
    W = w.shape[1]
    assert w.shape == (D, W)
    xp = _history(x, W, state_in)
    v = np.zeros((Bsz, D, L))
    for k in range(W):
        v += w[None, :, k, None] * xp[:, :, k:k + L]
    if bias is not None:
        v += bias[None, :, None]
    out = v * sigmoid(v) if silu else v.copy()
    return {"out": out, "pre": v, "state_out": xp[:, :, L:L + W - 1].copy()}


def conv_bwd(x, w, dout, bias=None, state_in=None, silu=True):
    """Gradient of <out, dout> w.r.t. x, w and bias: dict(dx, dw, dbias)."""
    x, w, dout = _f64(x), _f64(w), _f64(dout)
    Bsz, D, L = x.shape
    W = w.shape[1]
    f = conv_fwd(x, w, bias, state_in, silu)
    v = f["pre"]
    if silu:
        s = sigmoid(v)
        dv = dout * s * (1.0 + v * (1.0 - s))   # d/dv [v s(v)] = s + v s (1 - s)
    else:
        dv = dout.copy()
    xp = _history(x, W, state_in)
    dw = np.zeros((D, W))
    dxp = np.zeros_like(xp)
    for k in range(W):
        dw[:, k] = np.sum(dv * xp[:, :, k:k + L], axis=(0, 2))
        dxp[:, :, k:k + L] += w[None, :, k, None] * dv
    return {"dx": dxp[:, :, W - 1:], "dw": dw, "dbias": dv.sum(axis=(0, 2))}


def conv_step(state, x_t, w, bias=None, silu=True):
    """One token: state (B,D,W-1) oldest first, x_t (B,D).  Returns (out_t, new_state)."""
    state, x_t, w, bias = _f64(state), _f64(x_t), _f64(w), _f64(bias)
    W = w.shape[1]
    window = np.concatenate([state, x_t[:, :, None]], axis=2)          # (B,D,W)
    v = np.zeros_like(x_t)
    for k in range(W):
        v += w[None, :, k] * window[:, :, k]
    if bias is not None:
        v += bias[None, :]
    out = v * sigmoid(v) if silu else v
    return out, window[:, :, 1:].copy()
