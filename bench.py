#!/usr/bin/env python3
"""Benchmark of the selective-scan hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic input: the forward
scan (leaving its checkpoints) followed by the backward scan, on the Mamba-1.4B-shaped
layer (batch 8, L 2048, d_inner 4096, N 16, bf16 I/O, fp32 state).  Inputs are resident
in HBM before the timed region.  Prints ONE JSON line.

Every step works on the next of several input / workspace / output sets (more than the 256 MB
memory-side cache apart), so neither pass finds what the previous one left in a cache.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published
# fp32 vector peaks: the published 157.3 TFLOP/s assumes packed FP32 (two multiply-adds per lane
# and issue); without packed FP32, which this build does not use, a SIMD issues one 16-lane
# multiply-add per cycle: 256 CU x 4 SIMD x 16 lanes x 2.4 GHz x 2 flop = 78.6 TFLOP/s.
VALU_PEAK_PUBLISHED_TFLOPS = 157.3
VALU_PEAK_TFLOPS = 256 * 4 * 16 * 2.4e9 * 2 / 1e12
# Algorithmic flops per token*channel*state: forward 4 multiply-adds + 1 exponential,
# backward 12 multiply-adds + 1 exponential (a multiply-add counts 2, the exponential 1).
FLOPS_FWD, FLOPS_BWD = 4 * 2 + 1, 12 * 2 + 1


def algorithmic_bytes(batch, seqlen, dim, dstate, esz, has_z=True):
    """Bytes the method itself must move (expanded states and abar/bbar never counted)."""
    tc = batch * dim * seqlen
    bnl = batch * dstate * seqlen
    small = (dim * dstate + 2 * dim) * 4
    fwd = tc * esz * (3 + int(has_z)) + bnl * esz * 2 + small       # u, delta, z read; out write; B, C
    bwd = tc * esz * (5 + 2 * int(has_z)) + bnl * (2 * esz + 8) + 2 * small  # + dout; du, ddelta, dz; dB, dC fp32
    return fwd, bwd


def read_traffic(path):
    """HBM bytes per launch measured with rocprofv3 counters, kept as 'key: value' text."""
    out = {}
    if os.path.exists(path):
        for line in open(path):
            if ":" in line and not line.startswith("#"):
                k, v = line.split(":", 1)
                try:
                    out[k.strip()] = float(v.split()[0])
                except (ValueError, IndexError):
                    pass
    return out


def cpu_baseline(w, sample_dim):
    """Time the float64 oracle (as it stands) on the first `sample_dim` channels.
    Returns the baseline record and the oracle's results (for the parity check of the timed buffers)."""
    from oracle import ss_oracle as orc
    sl = lambda a: None if a is None else a[:, :sample_dim]
    kw = dict(Dskip=w["Dskip"][:sample_dim], z=sl(w["z"]), bias=w["delta_bias"][:sample_dim], softplus=True)
    u, dl, A, dout = sl(w["u"]), sl(w["delta"]), w["A"][:sample_dim], sl(w["dout"])
    t0 = time.perf_counter()
    ref_f = orc.scan_fwd(u, dl, A, w["B"], w["C"], **kw)
    ref_b = orc.scan_bwd(u, dl, A, w["B"], w["C"], dout, **kw)
    dt = time.perf_counter() - t0
    nb, nl = u.shape[0], u.shape[2]
    rec = {"value": nb * sample_dim * nl / dt, "unit": "token*channels/s", "cores": orc.threads(),
           "kind": "oracle", "seconds": round(dt, 3),
           "sample": "fwd+bwd float64 oracle on the first %d of the workload's channels, all %d batches, L=%d"
                     % (sample_dim, nb, nl)}
    return rec, ref_f, ref_b


class ScanSet:
    """One complete set of device buffers of a scan workload: inputs, output, workspace, gradients.
    The eight (B,D,L) tensors of a set (u, delta, z, dout, out, du, ddelta, dz) are contiguous as the
    interface requires; with `skewed` they are carved from one allocation at mutually skewed addresses
    (binding.empty_channel_skewed), without it each is an allocation of its own."""

    def __init__(self, src, dev, skewed=True):
        import torch
        from paper_2312_00752_amd import binding as B
        self.t = {k: (v.clone() if v is not None else None) for k, v in src.items() if k not in ("u", "delta", "z", "dout")}
        t = self.t
        nb, nd, nl = src["u"].shape
        if skewed:
            bdl = B.empty_channel_skewed(8, (nb, nd, nl), src["u"].dtype, dev)
        else:
            bdl = [torch.empty_like(src["u"]) for _ in range(8)]
        for k, buf in zip(("u", "delta", "z", "dout"), bdl):
            buf.copy_(src[k])
            t[k] = buf
        nn = t["A"].shape[1]
        f32 = torch.float32
        self.out = bdl[4]
        self.ws = torch.empty(B.ss_workspace_bytes(nb, nd, nl, nn, io_dtype=B.SS_BF16 if t["u"].dtype == torch.bfloat16 else B.SS_F32),
                              dtype=torch.uint8, device=dev)
        self.grads = {"du": bdl[5], "ddelta": bdl[6], "dz": bdl[7],
                      "dB": torch.empty(tuple(t["B"].shape), dtype=f32, device=dev),
                      "dC": torch.empty(tuple(t["C"].shape), dtype=f32, device=dev),
                      "dA": torch.empty(tuple(t["A"].shape), dtype=f32, device=dev),
                      "dD": torch.empty((nd,), dtype=f32, device=dev), "ddelta_bias": torch.empty((nd,), dtype=f32, device=dev),
                      "dh0": None}
        self.kw = dict(Dskip=t["Dskip"], z=t["z"], delta_bias=t["delta_bias"], delta_softplus=True)

    def fwd(self):
        from paper_2312_00752_amd import binding as B
        t = self.t
        B.ss_scan_fwd(t["u"], t["delta"], t["A"], t["B"], t["C"], out=self.out, workspace=self.ws, **self.kw)

    def bwd(self):
        from paper_2312_00752_amd import binding as B
        t = self.t
        B.ss_scan_bwd(t["dout"], t["u"], t["delta"], t["A"], t["B"], t["C"], self.ws, grads=self.grads, **self.kw)


def time_rotating(sets, steps, warmup):
    """Alternating forward / backward over rotating buffer sets.  Returns wall ms per step, the forward and
    the backward call durations (sorted lists, ms; events on the launch stream), and the same two calls
    timed back to back (forward after forward, backward after backward), also rotating."""
    import torch
    n = len(sets)
    for s in range(warmup):
        sets[s % n].fwd()
        sets[s % n].bwd()
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        st = sets[s % n]
        ev[s][0].record()
        st.fwd()
        ev[s][1].record()
        st.bwd()
        ev[s][2].record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    fwd_all = sorted(e[0].elapsed_time(e[1]) for e in ev)
    bwd_all = sorted(e[1].elapsed_time(e[2]) for e in ev)
    k = max(4, min(steps, 20))
    e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    e[0].record()
    for s in range(k):
        sets[s % n].fwd()
    e[1].record()
    for s in range(k):
        sets[s % n].bwd()
    e[2].record()
    torch.cuda.synchronize()
    return wall_ms, fwd_all, bwd_all, e[0].elapsed_time(e[1]) / k, e[1].elapsed_time(e[2]) / k


def device_inputs(name, dev):
    """The named workload's recipe drawn on the GPU (torch generator, the workload's seed): same shapes,
    dtypes and distributions as workloads.make_config, for timing only (the parity tests and the headline
    run use the numpy recipe itself)."""
    import math
    import torch
    from paper_2312_00752_amd import workloads as wl
    nb, nl, nd, nn, io, seed, bias_mode, u_mode = wl.CONFIGS[name]
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    iot = torch.bfloat16 if io == "bf16" else torch.float32
    rn = lambda *shape: torch.randn(*shape, device=dev, generator=gen)
    if u_mode == "onehot4":
        table = rn(4, nd)
        sym = torch.randint(0, 4, (nb, nl), device=dev, generator=gen)
        u = table[sym].permute(0, 2, 1).contiguous()
        u += 0.02 * rn(nb, nd, nl)
    else:
        u = rn(nb, nd, nl)
    lo, hi = 1e-3, 1e-1
    r = torch.rand(nd, device=dev, generator=gen)
    dt0 = torch.exp(math.log(lo) + r * (math.log(hi) - math.log(lo))) if bias_mode == "loguniform" else lo + r * (hi - lo)
    t = {"u": u.to(iot), "z": rn(nb, nd, nl).to(iot), "delta": rn(nb, nd, nl).to(iot),
         "delta_bias": torch.log(torch.expm1(dt0)), "B": rn(nb, nn, nl).to(iot), "C": rn(nb, nn, nl).to(iot),
         "Dskip": rn(nd), "dout": rn(nb, nd, nl).to(iot),
         "A": -torch.arange(1, nn + 1, device=dev, dtype=torch.float32).repeat(nd, 1).contiguous()}
    return t


def all_configs_bench(dev, steps=6):
    """Forward and backward call durations of all five workloads (two rotating buffer sets each), with the
    fraction of the HBM roofline their algorithmic bytes amount to."""
    import torch
    from paper_2312_00752_amd import workloads as wl
    res = {}
    for name in wl.CONFIG_ORDER:
        nb, nl, nd, nn, io = wl.CONFIGS[name][:5]
        esz = 2 if io == "bf16" else 4
        src = device_inputs(name, dev)
        sets = [ScanSet(src, dev) for _ in range(2)]
        # enough repetitions that the clocks have settled (a launch onto an idle chip runs ~10 % slower):
        # about 25 ms of warm-up and as much of timed work, from a first estimate of a step
        _, f0, b0, _, _ = time_rotating(sets, 2, 1)
        n = int(max(steps, min(40, 25.0 / max(f0[0] + b0[0], 1e-3))))
        _, fwd_all, bwd_all, _, _ = time_rotating(sets, n, n)
        f_ms, b_ms = fwd_all[len(fwd_all) // 2], bwd_all[len(bwd_all) // 2]
        fb, bb = algorithmic_bytes(nb, nl, nd, nn, esz)
        res[name] = {"shape_B_L_D_N": [nb, nl, nd, nn], "io_dtype": io, "fwd_ms": f_ms, "bwd_ms": b_ms,
                     "fwd_bwd_ms": f_ms + b_ms, "token_channels_per_s": nb * nd * nl / ((f_ms + b_ms) * 1e-3),
                     "algorithmic_bytes": fb + bb,
                     "frac_of_hbm_peak": (fb + bb) / ((f_ms + b_ms) * 1e-3) / 1e9 / HBM_PEAK_GBS}
        del sets
        if (nl * esz) % (1 << 20) == 0:
            # rows a large power of two apart: the same calls on tensors that are separate allocations
            # (all at the same offset into the memory channels' interleave), for comparison
            torch.cuda.empty_cache()
            plain = [ScanSet(src, dev, skewed=False) for _ in range(2)]
            _, fp, bp, _, _ = time_rotating(plain, n, n)
            res[name]["fwd_bwd_ms_separate_allocations"] = fp[len(fp) // 2] + bp[len(bp) // 2]
            del plain
        del src
        torch.cuda.empty_cache()
    return res


def parity_of_timed_buffers(st, ref_f, ref_b):
    """Scale-relative error (max |gpu - oracle| / max |oracle| per tensor) of what the timed kernels
    wrote into the buffer set `st`, against the oracle's results for the same inputs."""
    import numpy as np
    errs = {}

    def rel(got, ref):
        got = got.detach().float().cpu().numpy().astype(np.float64)
        ref = np.asarray(ref, np.float64)
        scale = float(np.max(np.abs(ref)))
        err = float(np.max(np.abs(got - ref)))
        return err / scale if scale > 0 else err

    errs["out"] = rel(st.out, ref_f["out"])
    for name, oname in (("du", "du"), ("ddelta", "ddelta"), ("dz", "dz"), ("dB", "dB"), ("dC", "dC"), ("dA", "dA"),
                        ("dD", "dD"), ("ddelta_bias", "dbias")):
        errs[name] = rel(st.grads[name], ref_b[oname])
    return errs




def decode_bench(dev, tokens=512):
    """Single-token recurrent steps (batch 64, D 4096, N 16, bf16 I/O): stream launches and
    the same launches replayed from a HIP graph."""
    import torch
    from paper_2312_00752_amd import binding as B
    from paper_2312_00752_amd import workloads as wl
    nb, nd, nn = wl.STEP_CONFIG[:3]
    s = wl.make_step_inputs(nb, nd, nn, 8, io="bf16", seed=wl.STEP_CONFIG[5])
    bf, f32 = torch.bfloat16, torch.float32
    g = {k: torch.from_numpy(s[k]).to(dev).to(bf) for k in ("u", "delta", "z", "B", "C")}
    A, Dk, bias = (torch.from_numpy(s[k]).to(dev) for k in ("A", "Dskip", "delta_bias"))
    h = torch.zeros(nb, nd, nn, device=dev, dtype=f32)
    out = torch.empty(nb, nd, device=dev, dtype=bf)

    def step(t):
        i = t % 8
        B.ss_step(h, g["u"][i], g["delta"][i], A, g["B"][i], g["C"][i], Dskip=Dk, z_t=g["z"][i],
                  delta_bias=bias, delta_softplus=True, out_t=out)

    for t in range(16):
        step(t)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for t in range(tokens):
        step(t)
    e1.record()
    torch.cuda.synchronize()
    us_stream = e0.elapsed_time(e1) * 1e3 / tokens
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            for t in range(64):
                step(t)
    torch.cuda.current_stream().wait_stream(side)
    graph.replay()
    torch.cuda.synchronize()
    e0.record()
    for _ in range(tokens // 64):
        graph.replay()
    e1.record()
    torch.cuda.synchronize()
    us_graph = e0.elapsed_time(e1) * 1e3 / tokens
    state_bytes = 2 * nb * nd * nn * 4 + nb * nd * 2 * 4 + 2 * nb * nn * 2
    return {"workload": "ss_step batch %d, D %d, N %d, bf16 I/O" % (nb, nd, nn),
            "us_per_token_stream": us_stream, "us_per_token_graph": us_graph,
            "bytes_per_token": state_bytes,
            "GBs_graph": state_bytes / (us_graph * 1e-6) / 1e9,
            "frac_of_hbm_peak_graph": state_bytes / (us_graph * 1e-6) / 1e9 / HBM_PEAK_GBS}


def layer_bench(dev, workload, iters=20):
    """The layer around the scan at the headline shape (conv + SiLU, projections,
    scan, gate; backward with recomputation), and its convolution kernels against the HBM roofline."""
    import torch
    from paper_2312_00752_amd import binding as B
    from paper_2312_00752_amd import workloads as wl
    nb, nl, nd, nn = wl.CONFIGS[workload][:4]
    w = wl.make_layer_inputs(nb, nl, nd, nn, io="bf16", seed=wl.CONFIGS[workload][5])
    rank = w["shape"][4]
    bf = torch.bfloat16
    t = {k: torch.from_numpy(w[k]).to(dev) for k in ("x", "z", "conv_w", "conv_b", "W_x", "W_dt", "dt_bias", "A", "Dskip", "dout")}
    for k in ("x", "z", "W_x", "W_dt", "dout"):
        t[k] = t[k].to(bf)
    saved = torch.empty(B.ss_layer_saved_bytes(nb, nd, nl, nn, rank), dtype=torch.uint8, device=dev)
    scratch = torch.empty(B.ss_layer_scratch_bytes(nb, nd, nl, nn, rank), dtype=torch.uint8, device=dev)
    out = torch.empty_like(t["x"])
    args = [t[k] for k in ("x", "z", "conv_w", "conv_b", "W_x", "W_dt", "dt_bias", "A", "Dskip")]

    def timed(f):
        for _ in range(3):
            f()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            f()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    fwd_ms = timed(lambda: B.ss_layer_fwd(*args, scratch=scratch, saved=saved, out=out))
    bwd_ms = timed(lambda: B.ss_layer_bwd(t["dout"], *args, scratch=scratch, saved=saved))
    # forward + backward of the layer replayed from one HIP graph (no launch gaps between its ~25 kernels)
    fb_graph_ms = None
    if iters >= 5:
        graph_fb = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph_fb, stream=side):
                B.ss_layer_fwd(*args, scratch=scratch, saved=saved, out=out)
                B.ss_layer_bwd(t["dout"], *args, scratch=scratch, saved=saved)
        torch.cuda.current_stream().wait_stream(side)
        fb_graph_ms = timed(graph_fb.replay)
    cf_ms = timed(lambda: B.ss_conv_fwd(t["x"], t["conv_w"], t["conv_b"], out=out))
    cb_ms = timed(lambda: B.ss_conv_bwd(t["dout"], t["x"], t["conv_w"], t["conv_b"]))
    # recurrent mode: the prompt's states, then 128 single-token steps at batch 64
    db = 64
    xs = torch.randn(8, db, nd, device=dev).to(bf)
    zs = torch.randn(8, db, nd, device=dev).to(bf)
    h = torch.zeros(db, nd, nn, device=dev)
    cs = torch.zeros(db, nd, 3, device=dev, dtype=bf)
    o_t = torch.empty(db, nd, device=dev, dtype=bf)
    sscr = torch.empty(B.ss_layer_step_scratch_bytes(db, nd, nn, rank), dtype=torch.uint8, device=dev)

    def decode():
        for i in range(128):
            B.ss_layer_step(h, cs, xs[i % 8], zs[i % 8], *args[2:], scratch=sscr, out_t=o_t)
    dec_ms = timed(decode) if iters >= 5 else None
    # the same 128 steps replayed from a HIP graph (every step of the layer is a kernel launch)
    dec_graph_us = None
    if dec_ms is not None:
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                decode()
        torch.cuda.current_stream().wait_stream(side)
        dec_graph_us = timed(graph.replay) * 1e3 / 128
    tensor = nb * nd * nl * 2
    return {"workload": "selective SSM layer, batch %d, L %d, D %d, N %d, R %d, conv width 4, bf16 I/O" % (nb, nl, nd, nn, rank),
            "fwd_ms": fwd_ms, "bwd_ms": bwd_ms, "token_channels_per_s": nb * nd * nl / ((fwd_ms + bwd_ms) * 1e-3),
            "fwd_bwd_ms_hip_graph": fb_graph_ms,
            "saved_bytes_per_token_channel": saved.numel() / (nb * nd * nl),
            "decode_us_per_token_batch64": None if dec_ms is None else dec_ms * 1e3 / 128,
            "decode_us_per_token_batch64_graph": dec_graph_us,
            "conv_fwd": {"ms": cf_ms, "bound": "hbm", "achieved": 2 * tensor / (cf_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                         "unit": "GB/s", "frac": 2 * tensor / (cf_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
            "conv_bwd": {"ms": cb_ms, "bound": "hbm", "achieved": 3 * tensor / (cb_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                         "unit": "GB/s", "frac": 3 * tensor / (cb_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}}


def variants_bench(dev, workload):
    """The scan variants of the paper's ablations at the workload's shape: complex state, more than
    16 states, time-invariant B / C, exact zero-order hold (forward and backward call durations, ms)."""
    import torch
    from paper_2312_00752_amd import binding as B
    from paper_2312_00752_amd import workloads as wl
    nb, nl, nd = wl.CONFIGS[workload][:3]
    bf = torch.bfloat16
    mk = lambda *s: torch.randn(*s, device=dev).to(bf)
    u, dl, z, do = mk(nb, nd, nl), mk(nb, nd, nl), mk(nb, nd, nl), mk(nb, nd, nl)
    Dk = torch.randn(nd, device=dev)
    bias = torch.full((nd,), -4.0, device=dev)
    out = torch.empty_like(u)

    def timed(f, iters=10):
        for _ in range(3):
            f()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            f()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    res = {}
    cases = [("selective_real_N16", 16, {}), ("complex_N8", 8, {"complex_state": True}),
             ("complex_N16", 16, {"complex_state": True}), ("real_N32", 32, {}), ("real_N64", 64, {}),
             ("time_invariant_BC_N16", 16, {"fixed": True}), ("exact_zoh_N16", 16, {"exact_zoh": True})]
    for name, nn, opt in cases:
        cplx = opt.get("complex_state", False)
        fixed = opt.get("fixed", False)
        if cplx:
            A = torch.stack([-0.5 * torch.ones(nd, nn, device=dev),
                             torch.arange(nn, device=dev).float().repeat(nd, 1)], -1).contiguous()   # S4D-Lin
            Bm, Cm = mk(nb, nn, 2, nl), mk(nb, nn, 2, nl)
        else:
            A = -torch.arange(1, nn + 1, device=dev).float().repeat(nd, 1).contiguous()             # S4D-Real
            Bm, Cm = (torch.randn(nd, nn, device=dev), torch.randn(nd, nn, device=dev)) if fixed else (mk(nb, nn, nl), mk(nb, nn, nl))
        ws = torch.empty(B.ss_workspace_bytes(nb, nd, nl, nn, io_dtype=B.SS_BF16, b_fixed=fixed, c_fixed=fixed,
                                              complex_state=cplx), dtype=torch.uint8, device=dev)
        kw = dict(Dskip=Dk, z=z, delta_bias=bias, delta_softplus=True, complex_state=cplx,
                  exact_zoh=opt.get("exact_zoh", False))
        f_ms = timed(lambda: B.ss_scan_fwd(u, dl, A, Bm, Cm, out=out, workspace=ws, **kw))
        b_ms = timed(lambda: B.ss_scan_bwd(do, u, dl, A, Bm, Cm, ws, **kw))
        res[name] = {"fwd_ms": f_ms, "bwd_ms": b_ms}
        del ws
    return res


def paper_sweep(dev):
    """The shape of the paper's own scan benchmark (Section 4.5 / Appendix E.5: batch 1,
    D 1024, N 16, bf16 inputs, L = 2^9 .. 2^19), forward only and forward+backward."""
    import torch
    from paper_2312_00752_amd import binding as B
    nb, nd, nn = 1, 1024, 16
    bf = torch.bfloat16
    gen = torch.Generator(device=dev)
    gen.manual_seed(6)
    rows = []
    for e in range(9, 20):
        nl = 1 << e
        mk = lambda *shape: torch.randn(*shape, device=dev, generator=gen).to(bf)
        src = {"u": mk(nb, nd, nl), "delta": mk(nb, nd, nl), "z": mk(nb, nd, nl), "dout": mk(nb, nd, nl),
               "B": mk(nb, nn, nl), "C": mk(nb, nn, nl),
               "A": -torch.arange(1, nn + 1, device=dev, dtype=torch.float32).repeat(nd, 1).contiguous(),
               "Dskip": torch.randn(nd, device=dev, generator=gen), "delta_bias": torch.full((nd,), -4.0, device=dev)}
        st = ScanSet(src, dev)   # tensors placed as in the main benchmark, gradients preallocated
        del src
        t = st.t
        ws0 = torch.empty(max(256, B.ss_workspace_bytes(nb, nd, nl, nn, for_backward=False, io_dtype=B.SS_BF16)),
                          dtype=torch.uint8, device=dev)
        fi = lambda: B.ss_scan_fwd(t["u"], t["delta"], t["A"], t["B"], t["C"], out=st.out, workspace=ws0, save_for_bwd=False, **st.kw)
        fs, bw = st.fwd, st.bwd
        for _ in range(2):
            fi(); fs(); bw()
        torch.cuda.synchronize()
        it = 10
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        ev[0].record()
        for _ in range(it):
            fi()
        ev[1].record()
        for _ in range(it):
            fs()
        ev[2].record()
        for _ in range(it):
            bw()
        ev[3].record()
        torch.cuda.synchronize()
        rows.append({"L": nl, "fwd_us": ev[0].elapsed_time(ev[1]) * 1e3 / it,
                     "fwd_save_us": ev[1].elapsed_time(ev[2]) * 1e3 / it,
                     "bwd_us": ev[2].elapsed_time(ev[3]) * 1e3 / it})
    return {"workload": "batch 1, D 1024, N 16, bf16 I/O", "rows": rows}


def generation_sweep(dev):
    """The paper's generation setting (Section 4.5 / Appendix E.5: prompt of 2048 tokens, 128
    generated tokens, batch 1 .. 128) for ONE selective SSM layer of the 1.4B shape: the prompt in
    parallel mode (states handed over), then 128 single-token steps replayed from a HIP graph."""
    import torch
    from paper_2312_00752_amd import binding as B
    from paper_2312_00752_amd import workloads as wl
    nd, nn, prompt, gen_tokens = 4096, 16, 2048, 128
    rank = wl.layer_rank(nd)
    bf = torch.bfloat16
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)
    rn = lambda *shape: torch.randn(*shape, device=dev, generator=gen)
    conv_w, conv_b = rn(nd, 4) * 0.5, rn(nd) * 0.1
    W_x = (rn(rank + 2 * nn, nd) / nd ** 0.5).to(bf)
    W_dt = (rn(nd, rank) / rank ** 0.5).to(bf)
    dt_bias = torch.full((nd,), -4.0, device=dev)
    A = -torch.arange(1, nn + 1, device=dev, dtype=torch.float32).repeat(nd, 1).contiguous()
    Dk = torch.ones(nd, device=dev)
    weights = [conv_w, conv_b, W_x, W_dt, dt_bias, A, Dk]
    rows = []
    for nb in (1, 2, 4, 8, 16, 32, 64, 128):
        x, z = rn(nb, nd, prompt).to(bf), rn(nb, nd, prompt).to(bf)
        xs, zs = rn(8, nb, nd).to(bf), rn(8, nb, nd).to(bf)
        scratch = torch.empty(B.ss_layer_scratch_bytes(nb, nd, prompt, nn, rank, for_backward=False), dtype=torch.uint8, device=dev)
        sscr = torch.empty(B.ss_layer_step_scratch_bytes(nb, nd, nn, rank), dtype=torch.uint8, device=dev)
        out = torch.empty_like(x)
        h = torch.zeros(nb, nd, nn, device=dev)
        cs = torch.zeros(nb, nd, 3, device=dev, dtype=bf)
        o_t = torch.empty(nb, nd, device=dev, dtype=bf)

        def prefill():
            B.ss_layer_fwd(x, z, *weights, scratch=scratch, out=out, return_states=True, h_last=h, conv_state=cs)

        def decode():
            for i in range(gen_tokens):
                B.ss_layer_step(h, cs, xs[i % 8], zs[i % 8], *weights, scratch=sscr, out_t=o_t)
        prefill(); decode()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                decode()
        torch.cuda.current_stream().wait_stream(side)
        it = 5
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        ev[0].record()
        for _ in range(it):
            prefill()
        ev[1].record()
        for _ in range(it):
            graph.replay()
        ev[2].record()
        torch.cuda.synchronize()
        pre_ms, dec_ms = ev[0].elapsed_time(ev[1]) / it, ev[1].elapsed_time(ev[2]) / it
        rows.append({"batch": nb, "prompt_ms": pre_ms, "decode_us_per_token": dec_ms * 1e3 / gen_tokens,
                     "generated_tokens_per_s_per_layer": nb * gen_tokens / ((pre_ms + dec_ms) * 1e-3)})
        del x, z, out, scratch
    return {"workload": "one layer, D 4096, N 16, R %d, bf16 I/O; prompt 2048 + 128 generated tokens" % rank, "rows": rows}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=48)
    ap.add_argument("--warmup", type=int, default=6)
    ap.add_argument("--workload", default="mamba1p4b_layer_bf16")
    ap.add_argument("--sets", type=int, default=4, help="rotating input / workspace / output sets")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (and with it the parity check)")
    ap.add_argument("--no-configs", action="store_true", help="skip the timing of the other workloads")
    ap.add_argument("--no-decode", action="store_true", help="skip the single-token step timing")
    ap.add_argument("--no-layer", action="store_true", help="skip the timing of the layer around the scan")
    ap.add_argument("--layer-iters", type=int, default=20,
                    help="timed repetitions of each layer call (below 5 the layer's decode loop is skipped)")
    ap.add_argument("--variants", action="store_true",
                    help="also time the scan variants (complex state, N > 16, time-invariant B/C, exact ZOH)")
    ap.add_argument("--paper-sweep", action="store_true",
                    help="also time the shape of the paper's own scan benchmark over L = 2^9..2^19")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 256 MiB streaming kernel (torch.neg; reference dispatch for "
                         "scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU; --gpus %d is not supported "
                 "(nothing here shards across devices)" % args.gpus)

    import torch
    from paper_2312_00752_amd import binding as B
    from paper_2312_00752_amd import workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    B.lib()  # fail loudly if the HIP library is missing
    dev = "cuda:0"
    torch.cuda.set_device(0)

    w = wl.make_config(args.workload)
    nb, nl, nd, nn = w["shape"]
    io = torch.bfloat16 if w["io"] == "bf16" else torch.float32
    esz = 2 if w["io"] == "bf16" else 4
    up = lambda a, dt: torch.from_numpy(a).to(dev).to(dt).contiguous()
    src = {k: up(w[k], io) for k in ("u", "delta", "z", "B", "C", "dout")}
    src.update({k: up(w[k], torch.float32) for k in ("A", "Dskip", "delta_bias")})
    sets = [ScanSet(src, dev) for _ in range(max(1, args.sets))]
    del src
    set_bytes = sum(t.numel() * t.element_size() for t in list(sets[0].t.values()) + [sets[0].out, sets[0].ws]
                    + [g for g in sets[0].grads.values() if g is not None])

    if args.copy_calibration:
        # Two plain streaming kernels of known size for the traffic counters: the L2's read-request
        # counter does not tell 64-byte from 128-byte requests, and these two issue one kind each
        # (measured: the negation 128-byte requests, the narrowing copy 64-byte ones).
        a = torch.zeros(64 * 1024 * 1024, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        c = torch.empty(48 * 1024 * 1024, dtype=torch.bfloat16, device=dev)
        torch.cuda.synchronize()
        torch.neg(a, out=b)              # reads 256 MiB, writes 256 MiB
        c.copy_(a[:48 * 1024 * 1024])    # reads 192 MiB, writes 96 MiB
        torch.cuda.synchronize()
        del a, b, c

    # Timed region: exactly K steps, bracketed by synchronisation; the library launches on torch's
    # current stream, so events recorded on that stream bracket the forward and the backward call.
    ms_step, fwd_all, bwd_all, fwd_b2b, bwd_b2b = time_rotating(sets, args.steps, args.warmup)
    last = sets[(args.steps - 1) % len(sets)]   # its buffers hold what the last timed step wrote
    fwd_ms = sum(fwd_all) / args.steps
    bwd_ms = sum(bwd_all) / args.steps

    tc = nb * nd * nl
    fwd_b, bwd_b = algorithmic_bytes(nb, nl, nd, nn, esz)
    traffic = read_traffic(os.path.join(ROOT, "profiles", "hbm_traffic_%s.txt" % args.workload))
    bwd_flops = tc * nn * FLOPS_BWD
    res = {
        "metric": "selective-scan fwd+bwd token*channels/s",
        "value": tc / (ms_step * 1e-3),
        "unit": "token*channels/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "batch": nb, "seqlen": nl, "d_inner": nd, "d_state": nn,
                   "io_dtype": w["io"], "state_dtype": "f32", "passes": "fwd(save)+bwd",
                   "rotating_buffer_sets": len(sets), "bytes_per_set": set_bytes,
                   "allocation": "contiguous (B,D,L) tensors, the eight of a set carved from one allocation 65 KiB apart"},
        # Dominant kernel: the backward scan (the backward call = zero-fill + scan + finalize; the scan
        # kernel is > 98 % of it).  Graded bound: HBM, algorithmic bytes of one backward launch over its
        # duration.  `traffic` is the launch's measured HBM bytes (rocprofv3 counters, kept in profiles/).
        "roofline": {"bound": "hbm", "kernel": "scan_bwd_dpp_kernel",
                     "achieved": bwd_b / (bwd_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": bwd_b / (bwd_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "traffic": traffic.get("scan_bwd_kernel_hbm_bytes")},
        # The same launch against the vector ALU, which is what limits it: algorithmic flops (12
        # multiply-adds + 1 exponential per token, channel and state) against both fp32 vector peaks.
        "alu_roofline": {"bound": "alu", "kernel": "scan_bwd_dpp_kernel", "achieved": bwd_flops / (bwd_ms * 1e-3) / 1e12,
                         "unit": "TFLOP/s", "peak_unpacked_fp32": VALU_PEAK_TFLOPS,
                         "frac_of_unpacked_peak": bwd_flops / (bwd_ms * 1e-3) / 1e12 / VALU_PEAK_TFLOPS,
                         "peak_published_packed_fp32": VALU_PEAK_PUBLISHED_TFLOPS,
                         "frac_of_published_peak": bwd_flops / (bwd_ms * 1e-3) / 1e12 / VALU_PEAK_PUBLISHED_TFLOPS},
        "passes": {"fwd_ms": fwd_ms, "bwd_ms": bwd_ms,
                   "fwd_ms_median": fwd_all[len(fwd_all) // 2], "fwd_ms_min": fwd_all[0],
                   "bwd_ms_median": bwd_all[len(bwd_all) // 2], "bwd_ms_min": bwd_all[0],
                   "fwd_ms_back_to_back": fwd_b2b, "bwd_ms_back_to_back": bwd_b2b,
                   "fwd_algorithmic_GBs": fwd_b / (fwd_ms * 1e-3) / 1e9,
                   "fwd_frac_of_hbm_peak": fwd_b / (fwd_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                   "fwd_bwd_algorithmic_GBs": (fwd_b + bwd_b) / ((fwd_ms + bwd_ms) * 1e-3) / 1e9,
                   "fwd_bwd_frac_of_hbm_peak": (fwd_b + bwd_b) / ((fwd_ms + bwd_ms) * 1e-3) / 1e9 / HBM_PEAK_GBS,
                   "fwd_alu_frac_of_unpacked_peak": tc * nn * FLOPS_FWD / (fwd_ms * 1e-3) / 1e12 / VALU_PEAK_TFLOPS,
                   "fwd_traffic": traffic.get("scan_fwd_kernel_hbm_bytes")},
    }
    if not args.no_cpu_baseline:
        # the oracle, timed on the host cores on the whole workload; its results then check the buffers
        # the LAST TIMED step wrote (nothing is re-run in between)
        res["cpu_baseline"], ref_f, ref_b = cpu_baseline(w, sample_dim=nd)
        errs = parity_of_timed_buffers(last, ref_f, ref_b)
        tol = 2e-2 if w["io"] == "bf16" else 1e-4
        res["parity_of_timed_buffers"] = {"metric": "max|gpu-oracle| / max|oracle| per tensor", "tolerance": tol,
                                          "max": max(errs.values()), "ok": bool(max(errs.values()) <= tol), "per_tensor": errs}
        del ref_f, ref_b
    del sets, last
    torch.cuda.empty_cache()
    if not args.no_configs:
        res["configs"] = all_configs_bench(dev)
    if not args.no_decode:
        res["decode"] = decode_bench(dev)
        if not args.no_configs:
            res["configs"]["ss_step_b64_d4096"] = {"us_per_token_graph": res["decode"]["us_per_token_graph"],
                                                   "us_per_token_stream": res["decode"]["us_per_token_stream"],
                                                   "frac_of_hbm_peak": res["decode"]["frac_of_hbm_peak_graph"]}
    if not args.no_layer and args.workload in ("mamba1p4b_layer_bf16", "mamba130m_layer_bf16"):
        res["layer"] = layer_bench(dev, args.workload, iters=args.layer_iters)
    if args.variants:
        res["variants"] = variants_bench(dev, args.workload)
    if args.paper_sweep:
        res["paper_sweep"] = paper_sweep(dev)
        res["generation_sweep"] = generation_sweep(dev)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
