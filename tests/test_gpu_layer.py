"""GPU parity of the selective SSM layer (conv, projections, scan, gate) against the float64 oracle.

For bf16 the oracle rounds the three intermediates the layer stores in bf16 (u, [r;B;C], delta_raw)
exactly where the layer does; everything else is float64."""
import numpy as np
import pytest

from oracle import inner_oracle as inn
from paper_2312_00752_amd.workloads import make_layer_inputs, round_to_bf16
from tests.util import assert_close

pytestmark = pytest.mark.gpu

PARAMS = ("x", "z", "conv_w", "conv_b", "W_x", "W_dt", "dt_bias", "A", "Dskip")
GRADS = {"dx": "dx", "dz": "dz", "dconv_w": "dconv_w", "dconv_b": "dconv_b", "dW_x": "dW_x", "dW_dt": "dW_dt",
         "ddt_bias": "ddt_bias", "dA": "dA", "dD": "dD"}


def _rnd(io):
    if io == "bf16":
        return lambda a: round_to_bf16(a).astype(np.float64)
    return lambda a: a.astype(np.float32).astype(np.float64)


def _gpu(w, backward=True):
    import torch
    from paper_2312_00752_amd import binding as B
    io = torch.bfloat16 if w["io"] == "bf16" else torch.float32
    t = {}
    for k in PARAMS + ("dout",):
        a = torch.from_numpy(np.ascontiguousarray(w[k])).cuda()
        t[k] = a.to(io) if k in ("x", "z", "W_x", "W_dt", "dout") else a
    batch, seqlen, dim, dstate, rank, width = w["shape"]
    code = B.SS_BF16 if w["io"] == "bf16" else B.SS_F32
    saved = torch.empty(B.ss_layer_saved_bytes(batch, dim, seqlen, dstate, rank, width, code), dtype=torch.uint8, device="cuda")
    scratch = torch.empty(B.ss_layer_scratch_bytes(batch, dim, seqlen, dstate, rank, width, code, True), dtype=torch.uint8, device="cuda")
    args = [t[k] for k in PARAMS]
    out = B.ss_layer_fwd(*args, scratch=scratch, saved=saved)
    # a forward call that keeps nothing gives the same result (same kernels, same order)
    out2 = B.ss_layer_fwd(*args, scratch=scratch)
    assert torch.equal(out, out2)
    g = None
    if backward:
        scratch.fill_(0x7f)   # nothing in the scratch buffer survives the forward call
        g = B.ss_layer_bwd(t["dout"], *args, scratch=scratch, saved=saved)
    torch.cuda.synchronize()
    return out, g


def _check(w, nthreads=0):
    out, g = _gpu(w)
    kw = {k: w[k] for k in PARAMS}
    ref = inn.inner_fwd(rnd=_rnd(w["io"]), nthreads=nthreads, **kw)
    assert_close(out, ref["out"], w["io"], "out", exact_inputs=False)
    rg = inn.inner_bwd(dout=w["dout"], rnd=_rnd(w["io"]), nthreads=nthreads, **kw)
    for name in GRADS:
        assert_close(g[name], rg[name], w["io"], name, exact_inputs=False)


@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(2, 200, 96, 16, 3), (1, 1031, 130, 8, 5), (2, 512, 256, 16, 8), (3, 77, 64, 4, 1)])
def test_layer_small(io, shape):
    batch, seqlen, dim, dstate, rank = shape
    _check(make_layer_inputs(batch, seqlen, dim, dstate, io, seed=seqlen, rank=rank))


# bf16 with R % 8 == 0 and L % 8 == 0: the forward scan projects delta itself, in contraction steps of
# 32 over R (4 or 8 of them), on whole and on split sequences, with ragged last chunks and channel groups
# The projection runs inside the scan only on unsplit sequences: 512 or more 64-row groups, or fewer than 128 steps
@pytest.mark.parametrize("shape", [(32, 264, 1024, 16, 160), (16, 200, 2048, 12, 256), (64, 136, 512, 16, 72),
                                   (32, 160, 1024, 16, 8), (5, 72, 320, 16, 64),
                                   # split sequences: the library GEMM
                                   (1, 2048, 128, 16, 160), (2, 1144, 100, 12, 136)])
def test_layer_projection_inside_scan(shape):
    batch, seqlen, dim, dstate, rank = shape
    w = make_layer_inputs(batch, seqlen, dim, dstate, "bf16", seed=rank, rank=rank)
    out, _ = _gpu(w, backward=False)
    ref = inn.inner_fwd(rnd=_rnd("bf16"), nthreads=0, **{k: w[k] for k in PARAMS})
    assert_close(out, ref["out"], "bf16", "out", exact_inputs=False)


def test_layer_narrow_conv_and_long_sequence():
    _check(make_layer_inputs(1, 4096, 128, 16, "bf16", seed=5, width=2))
    _check(make_layer_inputs(1, 2560, 64, 16, "f32", seed=6, width=3))


def test_layer_full_size_bf16():
    """The headline layer shape: batch 8, 2048 tokens, D = 4096, N = 16, R = 128."""
    _check(make_layer_inputs(8, 2048, 4096, 16, "bf16", seed=2))


# bf16 shapes with D % 32 == 0 and R % 8 == 0 take the hand-written matrix-core decode path (ragged
# batch tiles of 8 and of 16, ragged 64-channel groups, N below 16, R off and at the limits of the 32-wide
# contraction steps); the others take the library GEMMs
@pytest.mark.parametrize("io,shape", [("bf16", (4, 96, 256, 16, 8)), ("f32", (2, 40, 72, 5, 3)), ("bf16", (1, 33, 128, 16, 6)),
                                      ("bf16", (21, 40, 96, 8, 40)), ("bf16", (1, 20, 64, 16, 256)),
                                      ("bf16", (17, 24, 160, 12, 24)), ("bf16", (3, 20, 32, 16, 16)),
                                      ("f32", (3, 20, 64, 16, 8)),
                                      # more than 256 (channel group, 8-entry batch tile) pairs, at most 256
                                      # with 16-entry tiles: the wide tiles, last one ragged
                                      ("bf16", (234, 13, 1056, 16, 40)), ("bf16", (200, 14, 1088, 12, 24)),
                                      # more than 256 pairs either way: 8-entry tiles, two workgroups per CU
                                      ("bf16", (250, 13, 1056, 16, 40))])
def test_layer_prompt_then_token_by_token(io, shape):
    """Recurrent mode (Section 2): a prompt in parallel mode hands its states to single-token steps;
    the outputs must equal the parallel mode over the whole sequence."""
    import torch
    from paper_2312_00752_amd import binding as B
    batch, seqlen, dim, dstate, rank = shape
    w = make_layer_inputs(batch, seqlen, dim, dstate, io, seed=seqlen + 1, rank=rank)
    tio = torch.bfloat16 if io == "bf16" else torch.float32
    t = {}
    for k in PARAMS:
        a = torch.from_numpy(np.ascontiguousarray(w[k])).cuda()
        t[k] = a.to(tio) if k in ("x", "z", "W_x", "W_dt") else a
    code = B.SS_BF16 if io == "bf16" else B.SS_F32
    scratch = torch.empty(B.ss_layer_scratch_bytes(batch, dim, seqlen, dstate, rank, 4, code, False), dtype=torch.uint8, device="cuda")
    step_scratch = torch.empty(B.ss_layer_step_scratch_bytes(batch, dim, dstate, rank, code), dtype=torch.uint8, device="cuda")
    weights = [t[k] for k in PARAMS[2:]]
    cut = seqlen - 12
    head, h, cs = B.ss_layer_fwd(t["x"][:, :, :cut].contiguous(), t["z"][:, :, :cut].contiguous(), *weights,
                                 scratch=scratch, return_states=True)
    outs = [head]
    for i in range(cut, seqlen):
        o = B.ss_layer_step(h, cs, t["x"][:, :, i].contiguous(), t["z"][:, :, i].contiguous(), *weights, scratch=step_scratch)
        outs.append(o[:, :, None].clone())
    got = torch.cat(outs, 2)
    ref = inn.inner_fwd(rnd=_rnd(io), **{k: w[k] for k in PARAMS})
    assert_close(got[:, :, :cut], ref["out"][:, :, :cut], io, "prompt out", exact_inputs=False)
    assert_close(got[:, :, cut:], ref["out"][:, :, cut:], io, "decoded out", exact_inputs=False)
    assert_close(h, ref["h_last"], io, "h after decode", exact_inputs=False)
    np.testing.assert_array_equal(cs.float().cpu().numpy(), ref["conv_state"].astype(np.float32))


def test_layer_steps_replayed_from_a_hip_graph():
    """Decode steps captured once and replayed: every replay must equal the eager run."""
    import torch
    from paper_2312_00752_amd import binding as B
    batch, dim, dstate, rank, steps = 8, 256, 16, 8, 12
    w = make_layer_inputs(batch, steps, dim, dstate, "bf16", seed=41, rank=rank)
    bf = torch.bfloat16
    t = {}
    for k in PARAMS:
        a = torch.from_numpy(np.ascontiguousarray(w[k])).cuda()
        t[k] = a.to(bf) if k in ("x", "z", "W_x", "W_dt") else a
    xs = t["x"].permute(2, 0, 1).contiguous()
    zs = t["z"].permute(2, 0, 1).contiguous()
    weights = [t[k] for k in PARAMS[2:]]
    scratch = torch.empty(B.ss_layer_step_scratch_bytes(batch, dim, dstate, rank), dtype=torch.uint8, device="cuda")
    h = torch.zeros(batch, dim, dstate, device="cuda")
    cs = torch.zeros(batch, dim, 3, device="cuda", dtype=bf)
    outs = torch.empty(steps, batch, dim, device="cuda", dtype=bf)

    def run():
        for i in range(steps):
            B.ss_layer_step(h, cs, xs[i], zs[i], *weights, scratch=scratch, out_t=outs[i])
    run()                                   # eager, outside the capture
    torch.cuda.synchronize()
    want_out, want_h = outs.clone(), h.clone()
    ref = inn.inner_fwd(rnd=_rnd("bf16"), **{k: w[k] for k in PARAMS})
    assert_close(want_out.permute(1, 2, 0), ref["out"], "bf16", "eager decode", exact_inputs=False)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    h.zero_(); cs.zero_()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            run()
    torch.cuda.current_stream().wait_stream(side)
    for _ in range(3):
        h.zero_(); cs.zero_(); outs.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(outs, want_out) and torch.equal(h, want_h)
