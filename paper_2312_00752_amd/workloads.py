"""Seeded synthetic inputs for the selective scan.

This module holds no arithmetic of the method itself: it only draws the tensors that
both the GPU library and the CPU oracle are fed with.  The shapes stand in for the
paper's workloads (language-model layers of Table 12 at context 2048 with expansion 2,
Section 3.4; the million-token DNA setting of Section 4.3), whose data is not used.

Recipe (numpy ``default_rng(seed)``; draw order u, z, delta_raw, bias, B, C, Dskip, dout):
  u, z, delta_raw, B, C, Dskip, dout ~ N(0,1)
  A[d,n] = -(n+1)                                 (real S4D initialisation, Section 3.6)
  bias   = softplus^{-1}(U[1e-3, 1e-1])           (step-size initialisation, Section 3.6)
           ("loguniform": the step size itself is log-uniform on the same interval)
  u ("onehot4"): a random 4-symbol sequence embedded with a fixed random (4, D) table
           plus N(0, 0.02^2) noise
Tensors of a bf16 workload are rounded to bf16 once (round-to-nearest-even) and handed
out as float32 arrays holding exactly those values.

Layer recipe (``make_layer_inputs``; the block of Section 3.4 around the scan; draw order x, z,
conv_w, conv_b, W_x, W_dt, dt_bias, Dskip, dout):
  x, z, Dskip, dout ~ N(0,1)          (x, z stand for the two halves of the input projection)
  conv_w, conv_b ~ U[-W^-1/2, W^-1/2]  (width W = 4)
  W_x  (R+2N, D) ~ U[-D^-1/2, D^-1/2]  rows: Delta rank-R part, B, C   (Section 3.2, 3.6)
  W_dt (D, R)    ~ U[-R^-1/2, R^-1/2]  with R = ceil(D / 32)  (D/2 is the model width, R = width/16)
  dt_bias, A as above.
"""
import numpy as np

# name -> (batch, seqlen, dim, dstate, io dtype, seed, bias mode, u mode)
CONFIGS = {
    "tiny_fp32": (1, 256, 64, 16, "f32", 0, "uniform", "normal"),
    "mamba130m_layer_bf16": (8, 2048, 1536, 16, "bf16", 1, "uniform", "normal"),
    "mamba1p4b_layer_bf16": (8, 2048, 4096, 16, "bf16", 2, "uniform", "normal"),
    "mamba2p8b_long_bf16": (2, 16384, 5120, 16, "bf16", 3, "loguniform", "normal"),
    "genomics_1m_fp32": (1, 1048576, 256, 16, "f32", 4, "uniform", "onehot4"),
}
CONFIG_ORDER = list(CONFIGS)
# single-token decode workload: (batch, dim, dstate, io dtype, tokens, seed)
STEP_CONFIG = (64, 4096, 16, "bf16", 4096, 5)


def round_to_bf16(x):
    """Round a float32 array to the nearest bf16 value (ties to even); returns float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    rounded = (bits + np.uint32(0x7FFF) + ((bits >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def _inv_softplus(x):
    return np.log(np.expm1(x))


def make_scan_inputs(batch, seqlen, dim, dstate, io="f32", seed=0, bias_mode="uniform",
                     u_mode="normal", with_z=True, with_D=True, with_bias=True,
                     with_dout=True):
    """Return a dict of float32 numpy arrays (see the module docstring for the recipe)."""
    rng = np.random.default_rng(seed)
    shp = (batch, dim, seqlen)

    def normal(shape):
        return rng.standard_normal(shape, dtype=np.float32)

    if u_mode == "onehot4":
        table = normal((4, dim))
        u = np.empty(shp, dtype=np.float32)
        for b in range(batch):
            sym = rng.integers(0, 4, size=seqlen)
            u[b] = table[sym].T
            u[b] += np.float32(0.02) * normal((dim, seqlen))
    else:
        u = normal(shp)
    z = normal(shp)
    delta = normal(shp)
    lo, hi = 1e-3, 1e-1
    if bias_mode == "loguniform":
        dt0 = np.exp(rng.uniform(np.log(lo), np.log(hi), size=dim))
    else:
        dt0 = rng.uniform(lo, hi, size=dim)
    bias = _inv_softplus(dt0).astype(np.float32)
    Bm = normal((batch, dstate, seqlen))
    Cm = normal((batch, dstate, seqlen))
    Dskip = normal((dim,))
    dout = normal(shp) if with_dout else None
    A = -np.broadcast_to(np.arange(1, dstate + 1, dtype=np.float32), (dim, dstate)).copy()
    if io == "bf16":
        u, z, delta, Bm, Cm = (round_to_bf16(a) for a in (u, z, delta, Bm, Cm))
        if dout is not None:
            dout = round_to_bf16(dout)
    elif io != "f32":
        raise ValueError("io must be 'f32' or 'bf16'")
    out = {"u": u, "delta": delta, "A": A, "B": Bm, "C": Cm, "io": io,
           "shape": (batch, seqlen, dim, dstate), "delta_softplus": True}
    out["z"] = z if with_z else None
    out["Dskip"] = Dskip if with_D else None
    out["delta_bias"] = bias if with_bias else None
    out["dout"] = dout
    return out


def make_config(name, scale_batch=None, scale_seqlen=None, scale_dim=None, with_dout=True):
    """Inputs of a named workload; the ``scale_*`` arguments shrink a dimension while
    keeping the recipe (used by parity tests that the oracle must finish quickly)."""
    batch, seqlen, dim, dstate, io, seed, bias_mode, u_mode = CONFIGS[name]
    batch = scale_batch or batch
    seqlen = scale_seqlen or seqlen
    dim = scale_dim or dim
    w = make_scan_inputs(batch, seqlen, dim, dstate, io, seed, bias_mode, u_mode,
                         with_dout=with_dout)
    w["name"] = name
    return w


def make_step_inputs(batch, dim, dstate, tokens, io="bf16", seed=5):
    """Per-token decode inputs: u, delta, z (T,B,D); B, C (T,B,N); parameters as above."""
    rng = np.random.default_rng(seed)

    def normal(shape):
        return rng.standard_normal(shape, dtype=np.float32)

    u = normal((tokens, batch, dim))
    z = normal((tokens, batch, dim))
    delta = normal((tokens, batch, dim))
    bias = _inv_softplus(rng.uniform(1e-3, 1e-1, size=dim)).astype(np.float32)
    Bm = normal((tokens, batch, dstate))
    Cm = normal((tokens, batch, dstate))
    Dskip = normal((dim,))
    A = -np.broadcast_to(np.arange(1, dstate + 1, dtype=np.float32), (dim, dstate)).copy()
    if io == "bf16":
        u, z, delta, Bm, Cm = (round_to_bf16(a) for a in (u, z, delta, Bm, Cm))
    return {"u": u, "delta": delta, "z": z, "A": A, "B": Bm, "C": Cm, "Dskip": Dskip,
            "delta_bias": bias, "io": io, "shape": (batch, dim, dstate, tokens),
            "delta_softplus": True}


def make_conv_inputs(batch, dim, seqlen, width=4, io="bf16", seed=0):
    """Inputs of the short convolution: x, dout (B,D,L), state_in (B,D,W-1), w (D,W), bias (D)."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((batch, dim, seqlen), dtype=np.float32)
    dout = rng.standard_normal((batch, dim, seqlen), dtype=np.float32)
    state_in = rng.standard_normal((batch, dim, width - 1), dtype=np.float32)
    k = 1.0 / np.sqrt(width)
    w = rng.uniform(-k, k, size=(dim, width)).astype(np.float32)
    bias = rng.uniform(-k, k, size=dim).astype(np.float32)
    if io == "bf16":
        x, dout, state_in = round_to_bf16(x), round_to_bf16(dout), round_to_bf16(state_in)
    return {"x": x, "dout": dout, "state_in": state_in, "w": w, "bias": bias, "io": io,
            "shape": (batch, dim, seqlen, width)}


def layer_rank(dim):
    """Rank R of the Delta projection for an inner width ``dim`` (model width / 16, Section 3.6)."""
    return (dim + 31) // 32


def make_layer_inputs(batch, seqlen, dim, dstate=16, io="bf16", seed=0, width=4, rank=None):
    """Inputs of the selective SSM layer (see the module docstring for the recipe)."""
    rng = np.random.default_rng(seed)
    R = rank or layer_rank(dim)
    x = rng.standard_normal((batch, dim, seqlen), dtype=np.float32)
    z = rng.standard_normal((batch, dim, seqlen), dtype=np.float32)
    k = 1.0 / np.sqrt(width)
    conv_w = rng.uniform(-k, k, size=(dim, width)).astype(np.float32)
    conv_b = rng.uniform(-k, k, size=dim).astype(np.float32)
    k = 1.0 / np.sqrt(dim)
    W_x = rng.uniform(-k, k, size=(R + 2 * dstate, dim)).astype(np.float32)
    k = 1.0 / np.sqrt(R)
    W_dt = rng.uniform(-k, k, size=(dim, R)).astype(np.float32)
    dt_bias = _inv_softplus(rng.uniform(1e-3, 1e-1, size=dim)).astype(np.float32)
    Dskip = rng.standard_normal(dim, dtype=np.float32)
    dout = rng.standard_normal((batch, dim, seqlen), dtype=np.float32)
    A = -np.broadcast_to(np.arange(1, dstate + 1, dtype=np.float32), (dim, dstate)).copy()
    if io == "bf16":
        x, z, dout, W_x, W_dt = (round_to_bf16(a) for a in (x, z, dout, W_x, W_dt))
    return {"x": x, "z": z, "conv_w": conv_w, "conv_b": conv_b, "W_x": W_x, "W_dt": W_dt,
            "dt_bias": dt_bias, "A": A, "Dskip": Dskip, "dout": dout, "io": io,
            "shape": (batch, seqlen, dim, dstate, R, width)}
