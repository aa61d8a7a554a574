"""``torch.autograd`` front-ends of the library: the selective scan and the layer around it.

Still marshalling only: ``forward`` enqueues ``ss_scan_fwd`` / ``ss_layer_fwd`` and keeps the
workspace the library filled, ``backward`` enqueues ``ss_scan_bwd`` / ``ss_layer_bwd``; all
arithmetic happens in the HIP kernels.  Tensors use the library's layouts (sequence axis
last): u, delta, z (B,D,L); B, C (B,N,L) or a time-invariant (D,N) float32; A (D,N) float32.
"""
import torch

from . import binding as B


def _code(t):
    return B.SS_BF16 if t.dtype == torch.bfloat16 else B.SS_F32


class _SelectiveScan(torch.autograd.Function):
    @staticmethod
    def forward(ctx, u, delta, A, Bm, Cm, Dskip, z, delta_bias, h0, delta_softplus, exact_zoh, return_last_state):
        nb, nd, nl = u.shape
        nn = A.shape[1]
        ws = torch.empty(max(256, B.ss_workspace_bytes(nb, nd, nl, nn, True, _code(u), z is not None,
                                                       Bm.dim() == 2, Cm.dim() == 2)),
                         dtype=torch.uint8, device=u.device)
        out, h_last = B.ss_scan_fwd(u, delta, A, Bm, Cm, Dskip=Dskip, z=z, delta_bias=delta_bias, h0=h0,
                                    delta_softplus=delta_softplus, return_last_state=return_last_state,
                                    workspace=ws, save_for_bwd=True, exact_zoh=exact_zoh)
        ctx.save_for_backward(u, delta, A, Bm, Cm, Dskip, z, delta_bias, h0, ws)
        ctx.opts = (delta_softplus, exact_zoh)
        if return_last_state:
            return out, h_last
        return out

    @staticmethod
    def backward(ctx, dout, *rest):
        u, delta, A, Bm, Cm, Dskip, z, delta_bias, h0, ws = ctx.saved_tensors
        delta_softplus, exact_zoh = ctx.opts
        dh_last = rest[0] if rest and rest[0] is not None else None
        g = B.ss_scan_bwd(dout.contiguous(), u, delta, A, Bm, Cm, ws, Dskip=Dskip, z=z, delta_bias=delta_bias,
                          h0=h0, delta_softplus=delta_softplus,
                          dh_last=None if dh_last is None else dh_last.contiguous(),
                          want_dh0=h0 is not None, exact_zoh=exact_zoh)
        dB = g["dB"] if Bm.dim() == 2 else g["dB"].to(Bm.dtype)
        dC = g["dC"] if Cm.dim() == 2 else g["dC"].to(Cm.dtype)
        return (g["du"], g["ddelta"], g["dA"], dB, dC, g["dD"], g["dz"], g["ddelta_bias"], g["dh0"],
                None, None, None)


def selective_scan(u, delta, A, Bm, Cm, Dskip=None, z=None, delta_bias=None, h0=None, delta_softplus=False,
                   exact_zoh=False, return_last_state=False):
    """Differentiable selective scan (Algorithm 2, steps 5-6, with the gate of Section 3.4).
    Returns out, or (out, h_last) with ``return_last_state``."""
    return _SelectiveScan.apply(u, delta, A, Bm, Cm, Dskip, z, delta_bias, h0, delta_softplus, exact_zoh,
                                return_last_state)


class _SelectiveSSMLayer(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, z, conv_w, conv_b, W_x, W_dt, dt_bias, A, Dskip):
        nb, nd, nl = x.shape
        nn, rank, width = A.shape[1], W_dt.shape[1], conv_w.shape[1]
        code = _code(x)
        saved = torch.empty(B.ss_layer_saved_bytes(nb, nd, nl, nn, rank, width, code), dtype=torch.uint8, device=x.device)
        scratch = torch.empty(B.ss_layer_scratch_bytes(nb, nd, nl, nn, rank, width, code, False), dtype=torch.uint8,
                              device=x.device)
        out = B.ss_layer_fwd(x, z, conv_w, conv_b, W_x, W_dt, dt_bias, A, Dskip, scratch=scratch, saved=saved)
        ctx.save_for_backward(x, z, conv_w, conv_b, W_x, W_dt, dt_bias, A, Dskip, saved)
        return out

    @staticmethod
    def backward(ctx, dout):
        x, z, conv_w, conv_b, W_x, W_dt, dt_bias, A, Dskip, saved = ctx.saved_tensors
        nb, nd, nl = x.shape
        nn, rank, width = A.shape[1], W_dt.shape[1], conv_w.shape[1]
        scratch = torch.empty(B.ss_layer_scratch_bytes(nb, nd, nl, nn, rank, width, _code(x), True), dtype=torch.uint8,
                              device=x.device)
        g = B.ss_layer_bwd(dout.contiguous(), x, z, conv_w, conv_b, W_x, W_dt, dt_bias, A, Dskip, scratch=scratch,
                           saved=saved)
        return (g["dx"], g["dz"], g["dconv_w"], g["dconv_b"], g["dW_x"].to(W_x.dtype), g["dW_dt"].to(W_dt.dtype),
                g["ddt_bias"], g["dA"], g["dD"])


def selective_ssm_layer(x, z, conv_w, conv_b, W_x, W_dt, dt_bias, A, Dskip):
    """Differentiable layer around the scan: conv + SiLU, Delta/B/C projections, scan, gate (Section 3.4,
    Algorithm 2); only x, z, the small projection output and the scan's checkpoints are kept for backward."""
    return _SelectiveSSMLayer.apply(x, z, conv_w, conv_b, W_x, W_dt, dt_bias, A, Dskip)
