#!/usr/bin/env python3
"""Benchmark of the SSD forward+backward hot path under MA-GC on one MI355X.

One "step" = ssd_fwd + ssd_bwd (segment-by-segment restore) of one SSD layer over one batch of
seeded synthetic inputs that are already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--no-cpu-baseline]
"""
import argparse
import ctypes
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
VALU_FP32_PEAK_TFLOPS = 157.3


def kernel_models(cfg, tokens_per_launch, generic=False):
    """Algorithmic work of one launch of each kernel: (flop, bytes), MAC = 2 flop, dense Q x Q counts.
    Bytes are the tensors the step must read and write once (operands and results of that step; not
    the partial sums a launch configuration adds).  Per token, with X = H*P*e (one x-shaped tensor of
    element size e), S = H*P*N*2/Q (chunk states, bf16 in memory on the matrix-core path), R = 4H (one
    fp32 per-(token, head) array), b = G*N*e (B or C), g = G*Q*e (one row of the Q x Q matrix G):
      chunk_state   2NP*H   | x, cum, w, B -> states                      X + 2R + b + S
      cb            2QN*G   | B, C -> G and its transpose                 2b + 2g
      chunk_out  (2QP+2NP)H | x, states, G, C, cum, dt -> y               2X + S + g + b + 2R
      dstate_local  4NP*H   | x, dy, cum, w, B, C -> states, local adj.   2X + 2R + 2b + 2S
      bwd_main   (2QP+2NP)H | dy, x, adjoints, G^T, B, cum, dt -> dx + 3 scalar rows   3X + S + g + b + 5R
      dG            2QP*H   | x, dy, cum, dt, G -> dG, row-minus-column sums of E       2X + 2R + 2g + R
      dBC           4NP*H   | x, dy, states, adjoints, cum, w, B, C -> dB/dC state terms (fp32), two dot rows
                                                                          2X + 2S + 2R + 2b + 2*G*N*4 + 2R
      dBC_final     4QN*G   | dG, B, C, state terms -> dB, dC             g + 2b + 2*G*N*4 + 2b
      bwd_trio = bwd_main + dG + dBC as one launch (chunk 256): flop add up; x and dY count once
      state scans, per (chunk, head) state of P*N elements (matrix-core path, bf16 in memory):
      forward reads the chunk state and writes the entering state (4 B/element), reverse reads the
      local adjoint and the entering state and writes the total adjoint (6 B/element).
    A launch covers one segment: tokens_per_launch = batch * segment."""
    H, P, N, G, Q = cfg.nheads, cfg.headdim, cfg.dstate, cfg.ngroups, cfg.chunk
    t = tokens_per_launch
    esz = 2 if cfg.dtype == "bf16" else 4
    mfma = cfg.dtype == "bf16" and not generic   # the matrix-core path keeps only bf16 copies of the scanned states
    X, R, b, g = H * P * esz, 4 * H, G * N * esz, G * Q * esz
    S, S4 = H * P * N * 2 / Q, H * P * N * 4 / Q
    st = P * N * H / Q
    m = {
        "mfma_chunk_state": (2 * N * P * H, X + 2 * R + b + S), "mfma_cb": (2 * Q * N * G, 2 * b + 2 * g),
        "mfma_chunk_out": ((2 * Q * P + 2 * N * P) * H, 2 * X + S + g + b + 2 * R),
        "mfma_dstate_local": (4 * N * P * H, 2 * X + 2 * R + 2 * b + 2 * S),
        "mfma_bwd_main": ((2 * Q * P + 2 * N * P) * H, 3 * X + S + g + b + 5 * R),
        "mfma_dG": (2 * Q * P * H, 2 * X + 3 * R + 2 * g),
        "mfma_dBC": (4 * N * P * H, 2 * X + 2 * S + 4 * R + 2 * b + 8 * G * N),
        "mfma_dBC_final": (4 * Q * N * G, g + 4 * b + 8 * G * N),
        # bwd_main + dG + dBC in one launch (Q = 256): x and dY are read once for the three
        "mfma_bwd_trio": ((4 * Q * P + 6 * N * P) * H, 3 * X + 3 * S + 3 * g + 3 * b + 12 * R + 8 * G * N),
        # shape-generic fp32 FMA kernels (same operands; their states are fp32)
        "chunk_state": (2 * N * P * H, X + 2 * R + b + S4), "cb": (2 * Q * N * G, 2 * b + 2 * g),
        "chunk_out": ((2 * Q * P + 2 * N * P) * H, 2 * X + S4 + g + b + 2 * R),
        "dstate_local": (2 * N * P * H, X + R + b + S4),
        "bwd_main": ((4 * Q * P + 4 * N * P) * H, 3 * X + 2 * S4 + 2 * g + 2 * b + 5 * R),
        "dG": (2 * Q * P * H, 2 * X + 2 * R + g),
        "dBC": (4 * N * P * H + 4 * Q * N * G, 2 * X + 2 * S4 + 2 * R + g + 4 * b),
        "cumsum": (0, H * esz + 4 * 4 * H), "ddt_finalize": (0, 6 * 4 * H + H * esz),
        "state_scan_fwd": (0, (4 if mfma else 8) * st), "state_scan_bwd": (0, (6 if mfma else 12) * st),
    }
    return {k: (fl * t, by * t) for k, (fl, by) in m.items()}


def path_model(cfg):
    """Algorithmic work of the whole path per token of one layer (forward, restore, backward):
    flop = (2QP + 4NP)H + 2QN*G forward, twice that backward, (2NP)H + 2QN*G restore;
    bytes = forward reads x, dt, B, C and writes y; backward reads x, dt, B, C, dy and writes dx, ddt,
    dB, dC; the restore re-reads x, dt, B, C; the fp32 segment checkpoints are written and read once."""
    H, P, N, G, Q = cfg.nheads, cfg.headdim, cfg.dstate, cfg.ngroups, cfg.chunk
    esz = 2 if cfg.dtype == "bf16" else 4
    X, d, b = H * P * esz, H * esz, G * N * esz
    fwd_fl = (2 * Q * P + 4 * N * P) * H + 2 * Q * N * G
    flop = 3 * fwd_fl + 2 * N * P * H + 2 * Q * N * G
    byte = (2 * X + d + 2 * b) + (3 * X + 2 * d + 4 * b) + (X + d + 2 * b) + 2 * H * P * N * 4 / cfg.segment
    return flop, byte


def measured_traffic(kernel, workload):
    """HBM bytes per launch of `kernel` from the rocprofv3 --pmc runs summarised in profiles/traffic.json
    (FETCH_SIZE and WRITE_SIZE, scaled by a copy kernel of known size); None if not measured."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as f:
            return json.load(f).get(workload, {}).get(kernel)
    except (OSError, ValueError):
        return None


def cpu_baseline(cfg):
    """The fp64 oracle, as it stands, timed on this host on a bounded sample of the same workload: the first
    65536 tokens of every head (all of config 2), forward + backward, one run (about 10-20 s on 16 cores)."""
    from oracle import ssd_ref
    from paper_2411_19460_amd import synth
    threads = int(os.environ.get("OMP_NUM_THREADS", "0")) or (os.cpu_count() or 1)
    Ls = min(cfg.seqlen, 65536)
    sub = cfg.scaled(seqlen=Ls, segment=min(cfg.segment, Ls), name=cfg.name + "_sample")
    d = synth.make_layer_inputs(sub)
    t0 = time.perf_counter()
    ssd_ref.ssd_fwd(d["x"], d["dt"], d["A"], d["B"], d["C"], d["D"], None, sub.segment)
    ssd_ref.ssd_bwd(d["x"], d["dt"], d["A"], d["B"], d["C"], d["D"], d["dy"])
    dtm = time.perf_counter() - t0
    return {"value": sub.batch * Ls / dtm, "unit": "tokens/s", "cores": min(threads, cfg.nheads), "kind": "oracle",
            "seconds": dtm,
            "sample": f"first {Ls} tokens, all {cfg.nheads} heads, fwd+bwd fp64, one run (OpenMP over heads)"}


def inference_bench(args, cfg, pk, synth, torch, dev):
    """Forward-only use of the path: prefill of the whole sequence in segments without checkpoints
    (memory independent of L), then single-token recurrent steps from its final state."""
    d = synth.make_layer_inputs_device(cfg, dev, with_dy=False)
    Bt, L, H, P, N, G = cfg.batch, cfg.seqlen, cfg.nheads, cfg.headdim, cfg.dstate, cfg.ngroups
    shape = pk.make_shape(d["x"], d["B"], cfg.chunk, cfg.segment)
    ws = torch.empty(pk.ssd_workspace_bytes(shape, False), dtype=torch.uint8, device=dev)
    out = {"y": torch.empty_like(d["x"]), "final_state": torch.empty((Bt, H, P, N), device=dev)}

    def prefill():
        pk.ssd_fwd(d["x"], d["dt"], d["A"], d["B"], d["C"], d["D"], cfg.chunk, cfg.segment, None, 0, ws, out=out,
                   want_boundary=False)

    for _ in range(args.warmup):
        prefill()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        prefill()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    one = {k: d[k][:, :1].contiguous() for k in ("x", "dt", "B", "C")}
    y1 = torch.empty_like(one["x"])
    state = out["final_state"].clone()
    ntok = 200
    for _ in range(10):
        pk.ssd_decode(one["x"], one["dt"], d["A"], one["B"], one["C"], d["D"], state, out=y1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(ntok):
        pk.ssd_decode(one["x"], one["dt"], d["A"], one["B"], one["C"], d["D"], state, out=y1)
    torch.cuda.synchronize()
    us_tok = (time.perf_counter() - t0) * 1e6 / ntok
    esz = 2 if cfg.dtype == "bf16" else 4
    pre_bytes = (2 * H * P + H + 2 * G * N) * esz            # x, dt, B, C read, y written, per token
    dec_bytes = 2 * H * P * N * 4                            # fp32 state read and written, per token
    print(json.dumps({
        "metric": "SSD prefill tokens/sec/layer (forward only, no checkpoints)", "value": Bt * L / (ms * 1e-3),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name + "_prefill", "batch": Bt, "seqlen": L, "nheads": H, "headdim": P, "dstate": N,
                   "ngroups": G, "chunk": cfg.chunk, "segment": cfg.segment},
        "roofline": {"bound": "hbm", "achieved": pre_bytes * Bt * L / (ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": pre_bytes * Bt * L / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": None,
                     "note": "whole prefill: algorithmic bytes (x, dt, B, C read once, y written) over the step time"},
        "workspace_bytes": int(ws.numel()),
        "decode": {"us_per_token": us_tok, "tokens_per_call": 1, "state_bytes_per_token": dec_bytes,
                   "achieved_gbs": dec_bytes * Bt / (us_tok * 1e-6) / 1e9,
                   "note": "one launch per token from the host; bound by launch latency, not by the 5 MB of state"},
    }))


def conv_bench(args, cfg, pk, torch, dev):
    """Causal depthwise convolution (kernel 4) + SiLU of the block in front of the scan: channels =
    d_inner + 2 G N, one call over the whole sequence, forward then backward.  HBM-bound: the forward
    reads u and writes out, the backward reads u and dout and writes du (weights and states are noise)."""
    Bt, L = cfg.batch, cfg.seqlen
    C = cfg.nheads * cfg.headdim + 2 * cfg.ngroups * cfg.dstate
    g = torch.Generator(device=dev)
    g.manual_seed(cfg.seed(0) + 7)
    td = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    u = torch.randn((Bt, L, C), device=dev, generator=g, dtype=torch.float32).to(td)
    dout = torch.randn((Bt, L, C), device=dev, generator=g, dtype=torch.float32).to(td)
    w = torch.randn((C, 4), device=dev, generator=g) * 0.5
    bias = torch.randn((C,), device=dev, generator=g)
    st = torch.randn((Bt, 3, C), device=dev, generator=g, dtype=torch.float32).to(td)
    dso = torch.randn((Bt, 3, C), device=dev, generator=g)

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / args.steps

    ms_f = timed(lambda: pk.ssd_conv1d_fwd(u, w, bias, st))
    ms_b = timed(lambda: pk.ssd_conv1d_bwd(u, w, bias, st, dout, dso))
    esz = 2 if cfg.dtype == "bf16" else 4
    by_f, by_b = 2 * Bt * L * C * esz, 3 * Bt * L * C * esz
    print(json.dumps({
        "metric": "block conv1d+SiLU fwd+bwd tokens/sec/layer", "value": Bt * L / ((ms_f + ms_b) * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_f + ms_b, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name + "_conv1d", "batch": Bt, "seqlen": L, "channels": C},
        "roofline": {"bound": "hbm", "achieved": (by_f + by_b) / ((ms_f + ms_b) * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": (by_f + by_b) / ((ms_f + ms_b) * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": None,
                     "forward": {"ms": ms_f, "GB/s": by_f / (ms_f * 1e-3) / 1e9}, "backward": {"ms": ms_b, "GB/s": by_b / (ms_b * 1e-3) / 1e9}},
    }))


def norm_bench(args, cfg, pk, torch, dev):
    """Gated RMS normalisation of the block behind the scan: d_inner channels, one call over the whole
    sequence, forward then backward.  HBM-bound: the forward reads y and z and writes out, the backward
    reads y, z and dout and writes dy and dz."""
    T = cfg.batch * cfg.seqlen
    C = cfg.nheads * cfg.headdim
    g = torch.Generator(device=dev)
    g.manual_seed(cfg.seed(0) + 11)
    td = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    y, z, dout = (torch.randn((T, C), device=dev, generator=g, dtype=torch.float32).to(td) for _ in range(3))
    w = 1.0 + 0.3 * torch.randn((C,), device=dev, generator=g)
    dy, dz, dw = torch.empty_like(y), torch.empty_like(z), torch.empty_like(w)

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / args.steps

    ms_f = timed(lambda: pk.ssd_gated_norm_fwd(y, z, w, 1e-5, cfg.ngroups))
    ms_b = timed(lambda: pk.ssd_gated_norm_bwd(y, z, w, dout, 1e-5, cfg.ngroups, dy=dy, dz=dz, dw=dw))
    esz = 2 if cfg.dtype == "bf16" else 4
    by_f, by_b = 3 * T * C * esz, 5 * T * C * esz
    print(json.dumps({
        "metric": "block gated RMSNorm fwd+bwd tokens/sec/layer", "value": T / ((ms_f + ms_b) * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_f + ms_b, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name + "_gated_norm", "rows": T, "dim": C, "ngroups": cfg.ngroups},
        "roofline": {"bound": "hbm", "achieved": (by_f + by_b) / ((ms_f + ms_b) * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": (by_f + by_b) / ((ms_f + ms_b) * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": None,
                     "forward": {"ms": ms_f, "GB/s": by_f / (ms_f * 1e-3) / 1e9}, "backward": {"ms": ms_b, "GB/s": by_b / (ms_b * 1e-3) / 1e9}},
    }))


def linear_bench(args, cfg, pk, torch, dev):
    """The block's two projections at the config's width (d_model = d_inner / 2; the input projection
    widens to 2 d_inner + 2 G N + H, the output projection maps d_inner back), forward, input gradient
    and weight gradient over the whole sequence.  Dense contractions: priced against the bf16 matrix-core peak."""
    T = cfg.batch * cfg.seqlen
    d_inner = cfg.nheads * cfg.headdim
    d_model = d_inner // 2
    d_in_proj = 2 * d_inner + 2 * cfg.ngroups * cfg.dstate + cfg.nheads
    g = torch.Generator(device=dev)
    g.manual_seed(cfg.seed(0) + 13)
    rnd = lambda *s: torch.randn(s, device=dev, generator=g, dtype=torch.float32).to(torch.bfloat16)
    res = {}
    total_ms, total_flop = 0.0, 0.0
    for name, I, O in (("in_proj", d_model, d_in_proj), ("out_proj", d_inner, d_model)):
        x, w, dout = rnd(T, I), (rnd(O, I).float() / I ** 0.5).to(torch.bfloat16), rnd(T, O)
        out, dx, dw = torch.empty_like(dout), torch.empty_like(x), torch.empty((O, I), device=dev)

        def timed(fn):
            for _ in range(args.warmup):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3 / args.steps

        ms_f = timed(lambda: pk.ssd_linear_fwd(x, w, out))
        ms_dx = timed(lambda: pk.ssd_linear_bwd(x, w, dout, want_dw=False, dx=dx))
        ms_dw = timed(lambda: pk.ssd_linear_bwd(x, w, dout, want_dx=False, dw=dw))
        fl = 2.0 * T * I * O
        res[name] = {"in_dim": I, "out_dim": O, "forward": {"ms": ms_f, "TFLOP/s": fl / (ms_f * 1e-3) / 1e12},
                     "dx": {"ms": ms_dx, "TFLOP/s": fl / (ms_dx * 1e-3) / 1e12},
                     "dw": {"ms": ms_dw, "TFLOP/s": fl / (ms_dw * 1e-3) / 1e12}}
        total_ms += ms_f + ms_dx + ms_dw
        total_flop += 3 * fl
        del x, w, dout, out, dx, dw
    ach = total_flop / (total_ms * 1e-3) / 1e12
    print(json.dumps({
        "metric": "block projections fwd+bwd tokens/sec/layer", "value": T / (total_ms * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": total_ms, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": cfg.name + "_projections", "rows": T, "d_model": d_model, "d_in_proj": d_in_proj, "d_inner": d_inner},
        "roofline": {"bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": ach / MFMA_BF16_PEAK_TFLOPS, "traffic": None, **res},
    }))


def block_bench(args, cfg, pk, torch, dev):
    """One whole Mamba-2 block (projections, convolution, scan, gated norm) at the config's shape, forward
    + backward under sequence checkpoints every cfg.segment tokens.  The projections dominate (about 300 of
    the 316 MFLOP per token), so the step is priced against the bf16 matrix-core peak."""
    L, H, P, G, N = cfg.batch * cfg.seqlen, cfg.nheads, cfg.headdim, cfg.ngroups, cfg.dstate
    d_inner, dm = H * P, H * P // 2
    gn = G * N
    conv_dim, d_in_proj = d_inner + 2 * gn, 2 * d_inner + 2 * gn + H
    g = torch.Generator(device=dev)
    g.manual_seed(cfg.seed(0) + 17)
    rn = lambda *s: torch.randn(s, device=dev, generator=g, dtype=torch.float32)
    dt0 = torch.exp(torch.empty(H, device=dev).uniform_(math.log(1e-3), math.log(0.1), generator=g))
    par = {"W_in": (rn(d_in_proj, dm) / dm ** 0.5).to(torch.bfloat16), "conv_w": rn(conv_dim, 4) * 0.5, "conv_b": rn(conv_dim) * 0.2,
           "dt_bias": dt0 + torch.log(-torch.expm1(-dt0)), "A": -torch.exp(torch.empty(H, device=dev).uniform_(0.0, math.log(16.0), generator=g)),
           "D": rn(H), "norm_w": 1.0 + 0.3 * rn(d_inner), "W_out": (rn(dm, d_inner) / d_inner ** 0.5).to(torch.bfloat16)}
    if args.pre_norm:   # the language model's layer: RMS normalisation in front of the input projection
        par["pre_norm_w"] = 1.0 + 0.3 * rn(dm)
    u, dout = rn(L, dm).to(torch.bfloat16), rn(L, dm).to(torch.bfloat16)
    if args.layers > 1:
        # a stack of such blocks with residual adds on the two-axis grid: layer inputs kept every
        # --layer-interval layers, both states of every layer every cfg.segment tokens
        NL, li = args.layers, args.layer_interval
        layers = [par] + [{k: (v + 0.01 * torch.randn(v.shape, device=dev, generator=g, dtype=torch.float32).to(v.dtype)) if k in ("W_in", "W_out") else v.clone()
                           for k, v in par.items()} for _ in range(NL - 1)]
        if args.inference:
            # forward only, nothing kept: the prompt through all layers segment by segment, then one token per call
            st = {}

            def prefill():
                st.update(pk.magc_blockstack_infer(u, layers, H, P, G, N, cfg.chunk, cfg.segment, out=st.get("out"), workspace=st.get("workspace")))

            for _ in range(args.warmup):
                prefill()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                prefill()
            torch.cuda.synchronize()
            ms_p = (time.perf_counter() - t0) * 1e3 / args.steps
            # generation: the C entry point called directly with arguments marshalled once
            B = pk.binding
            pars = (B.magc_block_params_t * NL)(*[B.magc_block_params_t(*[(p[k].data_ptr() if k in p else None) for k in B.BLOCK_PARAMS]) for p in layers])
            one = B.magc_blockstack_shape_t(B.magc_block_shape_t(dm, H, P, G, N, cfg.chunk, 1e-5, 1, cfg.segment), NL, 1)
            tok = u[:1].clone()
            ws = torch.empty(int(pk.lib().magc_blockstack_workspace_bytes(ctypes.byref(one), 0)), dtype=torch.uint8, device=dev)
            stream = torch.cuda.current_stream().cuda_stream or None
            ntok = 32

            def generate():
                for _ in range(ntok):
                    rc = pk.lib().magc_blockstack_infer(ctypes.byref(one), pars, tok.data_ptr(), tok.data_ptr(), st["ssm_state"].data_ptr(),
                                                        st["conv_state"].data_ptr(), 0, ws.data_ptr(), ws.numel(), stream)
                    assert rc == 0, rc
            generate()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            generate()
            torch.cuda.synchronize()
            us_tok = (time.perf_counter() - t0) * 1e6 / ntok
            # the same step captured once in a graph and replayed (it enqueues kernels only)
            graph = torch.cuda.CUDAGraph()
            cap = torch.cuda.Stream()
            cap.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(cap):
                with torch.cuda.graph(graph, stream=cap):
                    rc = pk.lib().magc_blockstack_infer(ctypes.byref(one), pars, tok.data_ptr(), tok.data_ptr(), st["ssm_state"].data_ptr(),
                                                        st["conv_state"].data_ptr(), 0, ws.data_ptr(), ws.numel(), cap.cuda_stream)
                    assert rc == 0, rc
            torch.cuda.synchronize()
            for rep in range(2):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(ntok):
                    graph.replay()
                torch.cuda.synchronize()
                us_tok_graph = (time.perf_counter() - t0) * 1e6 / ntok
            # the same step for sixteen sequences at once: the parameters are read once for all of them
            nseq = 16
            ssm16 = torch.zeros((nseq, NL, H, P, N), dtype=torch.float32, device=dev)
            conv16 = torch.zeros((nseq, NL, 3, conv_dim), dtype=torch.bfloat16, device=dev)
            tok16 = u[:nseq].clone()

            def generate16():
                for _ in range(ntok):
                    rc = pk.lib().magc_blockstack_decode(ctypes.byref(one), pars, nseq, tok16.data_ptr(), tok16.data_ptr(), ssm16.data_ptr(),
                                                         conv16.data_ptr(), ws.data_ptr(), ws.numel(), stream)
                    assert rc == 0, rc
            generate16()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            generate16()
            torch.cuda.synchronize()
            us_step16 = (time.perf_counter() - t0) * 1e6 / ntok
            wbytes = sum(v.numel() * v.element_size() for v in par.values()) * NL
            print(json.dumps({
                "metric": "Mamba-2 block stack prefill tokens/sec/layer", "value": NL * L / (ms_p * 1e-3), "unit": "tokens/s", "n_gpus": 1,
                "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_p, "higher_is_better": True, "scaling": "weak",
                "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
                "config": {"workload": cfg.name + "_block_stack_prefill", "pre_norm": bool(args.pre_norm), "seqlen": L, "layers": NL,
                           "d_model": dm, "segment": cfg.segment},
                "roofline": {"bound": "mfma", "achieved": 2.0 * (dm * d_in_proj + d_inner * dm) * NL * L / (ms_p * 1e-3) / 1e12,
                             "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                             "frac": 2.0 * (dm * d_in_proj + d_inner * dm) * NL * L / (ms_p * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, "traffic": None},
                "generation": {"us_per_token": us_tok, "us_per_token_per_layer": us_tok / NL, "tokens": ntok,
                               "us_per_token_graph_replay": us_tok_graph,
                               "weights_and_states_bytes_per_token": wbytes + 2 * NL * H * P * N * 4,
                               "hbm_floor_us": (wbytes + 2 * NL * H * P * N * 4) / HBM_PEAK_GBS / 1e3,
                               "note": "one C call per token; every parameter read once and every SSM state read and written once per token"},
                "batched_generation": {"sequences": nseq, "us_per_step": us_step16, "us_per_step_per_layer": us_step16 / NL,
                                       "tokens_per_s": nseq / (us_step16 * 1e-6),
                                       "hbm_floor_us": (wbytes + 2 * nseq * NL * H * P * N * 4) / HBM_PEAK_GBS / 1e3,
                                       "note": "one token for each of the sequences per call (magc_blockstack_decode)"},
                "workspace_bytes": int(ws.numel()),
            }))
            return
        grads = [{"d" + k: torch.empty(v.shape, dtype=torch.float32, device=dev) for k, v in par.items()} for _ in range(NL)]
        f = {}

        def sfwd():
            f.update(pk.magc_blockstack_fwd(u, layers, H, P, G, N, cfg.chunk, cfg.segment, li))

        def sbwd():
            pk.magc_blockstack_bwd(u, layers, dout, f["l_ckpt"], f["ssm_ckpt"], f["conv_ckpt"], H, P, G, N, cfg.chunk, cfg.segment, li, grads=grads)

        def timed(fn):
            for _ in range(args.warmup):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3 / args.steps

        ms_f, ms_b = timed(sfwd), timed(sbwd)
        assert bool(torch.isfinite(grads[0]["dW_in"].sum())) and bool(torch.isfinite(f["out"].float().sum()))
        sshp = pk.binding.magc_blockstack_shape_t(pk.binding.magc_block_shape_t(dm, H, P, G, N, cfg.chunk, 1e-5, L, cfg.segment), NL, li)
        nseg, ngl = -(-L // cfg.segment), -(-NL // li)
        kept = NL * nseg * (H * P * N * 4 + 3 * conv_dim * 2) + (ngl - 1) * L * dm * 2
        print(json.dumps({
            "metric": "Mamba-2 block stack fwd+bwd tokens/sec/layer", "value": NL * L / ((ms_f + ms_b) * 1e-3), "unit": "tokens/s",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_f + ms_b, "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": cfg.name + "_block_stack", "pre_norm": bool(args.pre_norm), "seqlen": L, "layers": NL, "layer_interval": li, "d_model": dm,
                       "segment": cfg.segment},
            "roofline": {"bound": "mfma", "achieved": None, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": None, "traffic": None,
                         "forward_ms": ms_f, "backward_ms": ms_b},
            "peak_hbm": {"checkpoint_bytes": kept, "workspace_bytes": int(pk.lib().magc_blockstack_workspace_bytes(ctypes.byref(sshp), 1)),
                         "per_layer_input_bytes": NL * L * dm * 2,
                         "note": "kept between the passes: state checkpoints of every layer + layer inputs every layer_interval layers; "
                                 "per_layer_input_bytes is what keeping every layer's input (plain per-layer checkpointing) would hold"},
        }))
        return
    if args.inference:
        # forward only, no checkpoint kept: the prompt in segments, then one token per call from the carried states
        def prefill():
            return pk.magc_block_fwd(u, par, H, P, G, N, cfg.chunk, cfg.segment, checkpoints=False)
        for _ in range(args.warmup):
            prefill()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            f = prefill()
        torch.cuda.synchronize()
        ms_p = (time.perf_counter() - t0) * 1e3 / args.steps
        ntok = 64
        tok = u[:1].contiguous()
        for rep in range(2):   # the second pass is the timed one
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            st = f
            for _ in range(ntok):
                st = pk.magc_block_fwd(tok, par, H, P, G, N, cfg.chunk, cfg.segment, init_ssm=st["final_ssm"],
                                       init_conv=st["final_conv"], checkpoints=False)
            torch.cuda.synchronize()
            us_tok = (time.perf_counter() - t0) * 1e6 / ntok
        shp = pk.binding.magc_block_shape_t(dm, H, P, G, N, cfg.chunk, 1e-5, L, cfg.segment)
        print(json.dumps({
            "metric": "Mamba-2 block prefill tokens/sec/layer", "value": L / (ms_p * 1e-3), "unit": "tokens/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_p, "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": cfg.name + "_block_prefill", "seqlen": L, "d_model": dm, "segment": cfg.segment},
            "roofline": {"bound": "mfma", "achieved": 2.0 * (dm * d_in_proj + d_inner * dm) * L / (ms_p * 1e-3) / 1e12,
                         "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": 2.0 * (dm * d_in_proj + d_inner * dm) * L / (ms_p * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, "traffic": None},
            "generation": {"us_per_token": us_tok, "tokens": ntok, "note": "one call per token from the host: two weight-streaming products and the recurrence kernel (plus one state copy)"},
            "workspace_bytes": int(pk.lib().magc_block_workspace_bytes(ctypes.byref(shp), 0)),
        }))
        return
    grads = {"d" + k: torch.empty(v.shape, dtype=torch.float32, device=dev) for k, v in par.items()}
    f = {}

    def fwd():
        f.update(pk.magc_block_fwd(u, par, H, P, G, N, cfg.chunk, cfg.segment))

    def bwd():
        pk.magc_block_bwd(u, par, dout, f["ssm_ckpt"], f["conv_ckpt"], H, P, G, N, cfg.chunk, cfg.segment, grads=grads)

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / args.steps

    ms_f, ms_b = timed(fwd), timed(bwd)
    assert bool(torch.isfinite(grads["dW_in"].sum())) and bool(torch.isfinite(f["out"].float().sum()))
    proj = 2.0 * (dm * d_in_proj + d_inner * dm)                       # per token, forward
    ssd_f = (2 * cfg.chunk * P + 4 * N * P) * H + 2 * cfg.chunk * N * G   # the scan's forward contractions per token
    # forward; input and weight gradients; the recomputed input projection; the scan forward, recomputed, backward
    flop_tok = proj + 2 * proj + 2.0 * dm * d_in_proj + 4 * ssd_f
    ach = flop_tok * L / ((ms_f + ms_b) * 1e-3) / 1e12
    shp = pk.binding.magc_block_shape_t(dm, H, P, G, N, cfg.chunk, 1e-5, L, cfg.segment)
    full = pk.binding.magc_block_shape_t(dm, H, P, G, N, cfg.chunk, 1e-5, L, L)
    nseg = -(-L // cfg.segment)
    ckpt = nseg * (H * P * N * 4 + 3 * conv_dim * 2)
    print(json.dumps({
        "metric": "Mamba-2 block fwd+bwd tokens/sec/layer", "value": L / ((ms_f + ms_b) * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_f + ms_b, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": cfg.name + "_block", "pre_norm": bool(args.pre_norm), "seqlen": L, "d_model": dm, "nheads": H, "headdim": P, "ngroups": G, "dstate": N,
                   "chunk": cfg.chunk, "segment": cfg.segment},
        "roofline": {"bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": ach / MFMA_BF16_PEAK_TFLOPS,
                     "traffic": None, "flop_per_token": flop_tok, "forward_ms": ms_f, "backward_ms": ms_b},
        "peak_hbm": {"magc_bytes": int(pk.lib().magc_block_workspace_bytes(ctypes.byref(shp), 1)) + ckpt,
                     "full_activation_bytes": int(pk.lib().magc_block_workspace_bytes(ctypes.byref(full), 1)),
                     "note": "workspace + checkpoints beyond inputs, outputs and parameter gradients: checkpoints every "
                             "segment vs one segment = the whole sequence (every activation of the block alive)"},
    }))


# Kernel -> the part of the path whose inputs and outputs it moves.  The algorithmic bytes of a part are the
# tensors the method must read and write there once per token (bf16 storage: x-shaped tensors H*P*e, dt-shaped
# H*e, B/C-shaped G*N*e): forward reads x, dt, B, C and writes y; the restore of a segment re-reads x, dt, B, C;
# backward reads x, dt, B, C, dy and writes dx, ddt, dB, dC.
KERNEL_GROUP = {"cumsum": "fwd", "mfma_cb": "fwd", "cb": "fwd", "mfma_chunk_state": "fwd", "chunk_state": "fwd",
                "state_scan_fwd": "fwd", "mfma_chunk_out": "fwd", "chunk_out": "fwd",
                "mfma_dstate_local": "restore", "dstate_local": "restore",
                "state_scan_bwd": "bwd", "mfma_bwd_trio": "bwd", "mfma_bwd_main": "bwd", "bwd_main": "bwd", "mfma_dG": "bwd",
                "dG": "bwd", "mfma_dBC": "bwd", "dBC": "bwd", "mfma_dBC_final": "bwd", "ddt_finalize": "bwd"}


def group_bytes(cfg):
    H, P, N, G = cfg.nheads, cfg.headdim, cfg.dstate, cfg.ngroups
    e = 2 if cfg.dtype == "bf16" else 4
    X, d, b = H * P * e, H * e, G * N * e
    return {"fwd": 2 * X + d + 2 * b, "restore": X + d + 2 * b, "bwd": 3 * X + 2 * d + 4 * b}


def measured_peak(torch, fn):
    """Device bytes allocated at the peak of fn() beyond what was allocated when it started, and fn's result."""
    torch.cuda.synchronize()
    base = torch.cuda.memory_allocated()
    torch.cuda.reset_peak_memory_stats()
    out = fn()
    torch.cuda.synchronize()
    return torch.cuda.max_memory_allocated() - base, out


def layer_bench(cfg, steps, warmup, flags, pk, synth, torch, dev, per_kernel, measure_peak=True):
    """ssd_fwd + ssd_bwd of one layer on inputs resident in HBM: wall clock over exactly `steps` steps, the
    median over the steps (an event between steps), the measured peak of device memory beyond inputs and
    outputs for MA-GC and for one segment = the whole sequence, and, on request, the per-kernel table."""
    d = synth.make_layer_inputs_device(cfg, dev)
    ck_dtype = torch.bfloat16 if flags & pk.SSD_FLAG_BF16_CHECKPOINTS else torch.float32
    Bt, L, H, P, N = cfg.batch, cfg.seqlen, cfg.nheads, cfg.headdim, cfg.dstate
    nseg = -(-L // cfg.segment)
    out_f = {"y": torch.empty_like(d["x"]), "final_state": torch.empty((Bt, H, P, N), device=dev)}
    out_b = {"dx": torch.empty_like(d["x"]), "ddt": torch.empty_like(d["dt"]), "dB": torch.empty_like(d["B"]),
             "dC": torch.empty_like(d["C"]), "dinit_state": torch.empty((Bt, H, P, N), device=dev)}
    dA = torch.empty(H, device=dev)
    dD = torch.empty(H, device=dev)

    def one_pass(segment):
        # everything beyond the inputs and the outputs is allocated inside: checkpoints and both workspaces
        _, _, bnd = pk.ssd_fwd(d["x"], d["dt"], d["A"], d["B"], d["C"], d["D"], cfg.chunk, segment, None, flags, None, out=out_f)
        pk.ssd_bwd(d["x"], d["dt"], d["A"], d["B"], d["C"], d["D"], d["dy"], cfg.chunk, segment, None, None, bnd, flags,
                   None, dA, dD, out=out_b)

    one_pass(cfg.segment)          # warm: library streams and events exist, code objects are loaded
    peak_magc = peak_full = None
    if measure_peak:
        peak_magc, _ = measured_peak(torch, lambda: one_pass(cfg.segment))
        peak_full, _ = measured_peak(torch, lambda: one_pass(None))
    torch.cuda.empty_cache()
    shape = pk.make_shape(d["x"], d["B"], cfg.chunk, cfg.segment)
    peak_hbm = {"magc_bytes": peak_magc, "full_activation_bytes": peak_full,
                "magc_formula_bytes": pk.ssd_workspace_bytes(shape, True, flags) + nseg * Bt * H * P * N * (2 if ck_dtype == torch.bfloat16 else 4),
                "note": "torch.cuda.max_memory_allocated during ssd_fwd + ssd_bwd minus what was allocated before (inputs "
                        "and outputs): checkpoints + workspaces.  MA-GC (checkpoint every segment, scratch of the segments "
                        "in flight) vs one segment = the whole sequence (every chunk state of the sequence alive)"}

    ws_f = torch.empty(pk.ssd_workspace_bytes(shape, False, flags), dtype=torch.uint8, device=dev)
    ws_b = torch.empty(pk.ssd_workspace_bytes(shape, True, flags), dtype=torch.uint8, device=dev)
    out_f["boundary_states"] = torch.empty((Bt, nseg, H, P, N), dtype=ck_dtype, device=dev)

    def step():
        pk.ssd_fwd(d["x"], d["dt"], d["A"], d["B"], d["C"], d["D"], cfg.chunk, cfg.segment, None, flags, ws_f, out=out_f)
        pk.ssd_bwd(d["x"], d["dt"], d["A"], d["B"], d["C"], d["D"], d["dy"], cfg.chunk, cfg.segment, None, None,
                   out_f["boundary_states"], flags, ws_b, dA, dD, out=out_b)

    for _ in range(warmup):
        step()
    # the timed region: exactly `steps` steps, nothing but the calls and one event record between steps
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(steps):
        step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    step_ms = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(steps))
    median = step_ms[len(step_ms) // 2] if len(step_ms) % 2 else 0.5 * (step_ms[len(step_ms) // 2 - 1] + step_ms[len(step_ms) // 2])
    res = {"tokens_per_s": Bt * L / (ms_per_step * 1e-3), "ms_per_step": ms_per_step, "median_ms_per_step": median,
           "step_ms": step_ms, "peak_hbm": peak_hbm}
    if not per_kernel:
        return res
    # Untimed pass 1: every segment on one stream, HIP events around every launch: the per-kernel table.
    pk.ssd_prof_serialize(True)
    pk.ssd_prof_enable(True)
    nser = 3
    for _ in range(nser):
        step()
    torch.cuda.synchronize()
    prof_all = pk.ssd_prof_read()
    pk.ssd_prof_enable(False)
    pk.ssd_prof_serialize(False)
    models = kernel_models(cfg, Bt * cfg.segment, bool(flags & pk.SSD_FLAG_GENERIC_KERNELS))
    kernels = {}
    for name, (ms, n) in prof_all.items():
        ent = {"ms_per_step": ms / nser, "launches_per_step": n // nser, "avg_us": ms * 1e3 / n}
        if name in models:
            fl, by = models[name]
            sec = ms / n * 1e-3
            ent["operand_gbs"] = by / sec / 1e9       # operands and results of this kernel alone (states and scores included)
            if fl:
                ent["tflops"] = fl / sec / 1e12
        kernels[name] = ent
    dom = max((k for k in kernels if k in models), key=lambda k: kernels[k]["ms_per_step"])
    # Untimed pass 2: as the timed region (segments in flight), events around the dominant kernel only.
    step()
    pk.ssd_prof_enable(True, only=dom)
    for _ in range(nser):
        step()
    torch.cuda.synchronize()
    pd = pk.ssd_prof_read()
    pk.ssd_prof_enable(False)
    res.update({"kernels_serialized": kernels, "dominant": dom,
                "dominant_in_flight_us": pd[dom][0] * 1e3 / pd[dom][1] if dom in pd else None})
    return res


def stack_bench(cfg, steps, warmup, pk, synth, torch, dev):
    """The 16-layer residual stack on its MA-GC grid (all layers x cfg.segment tokens per cell): forward + backward
    tokens/s per layer and the measured peak of device memory beyond inputs and outputs, against the same stack
    under layer-only checkpointing (every layer's input kept for the whole sequence, no sequence checkpoints)."""
    layers = []
    for j in range(cfg.nlayers):
        lay = synth.make_layer_inputs_device(cfg, dev, layer=j, with_dy=(j == 0))
        if j == 0:
            x0, dout = lay["x"], lay["dy"]
        layers.append({k: lay[k] for k in ("dt", "A", "B", "C", "D")})
        del lay
    stk = [torch.stack([l[k] for l in layers]).contiguous() for k in ("dt", "A", "B", "C", "D")]
    del layers
    torch.cuda.empty_cache()
    nl, L = cfg.nlayers, cfg.seqlen

    def one(segment, interval):
        f = pk.magc_stack_fwd(x0, *stk, cfg.chunk, segment, interval, want_final=False)
        b = pk.magc_stack_bwd(x0, *stk, dout, f["s_ckpt"], f["l_ckpt"], cfg.chunk, segment, interval)
        return f["out"].numel() * f["out"].element_size() + sum(v.numel() * v.element_size() for v in b.values())

    def arm(segment, interval):
        for _ in range(warmup):
            one(segment, interval)
        peak, out_bytes = measured_peak(torch, lambda: one(segment, interval))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            one(segment, interval)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        torch.cuda.empty_cache()
        # the outputs (out, dx0 and the per-layer gradients) are allocated inside the call: not part of the figure
        return {"ms_per_step": ms, "tokens_per_s_per_layer": nl * cfg.batch * L / (ms * 1e-3), "peak_bytes": peak - out_bytes}

    grid = arm(cfg.segment, nl)
    layer_only = arm(L, 1)
    return {"nlayers": nl, "seqlen": L, "segment": cfg.segment, "layer_interval": nl,
            "tokens_per_s_per_layer": grid["tokens_per_s_per_layer"], "ms_per_step": grid["ms_per_step"],
            "peak_hbm": {"magc_grid_bytes": grid["peak_bytes"], "layer_only_bytes": layer_only["peak_bytes"],
                         "note": "torch.cuda.max_memory_allocated during magc_stack_fwd + magc_stack_bwd minus inputs and "
                                 "outputs: checkpoints + workspace.  Grid of all layers x segment tokens vs every layer input "
                                 "kept for the whole sequence with one segment = the whole sequence"},
            "layer_only": {"tokens_per_s_per_layer": layer_only["tokens_per_s_per_layer"], "ms_per_step": layer_only["ms_per_step"]}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=2, help="index into the benchmark's config list (default: 2.7B shape, L=65536)")
    ap.add_argument("--segment", type=int, default=0, help="checkpoint interval in tokens (default: the config's)")
    ap.add_argument("--generic", action="store_true", help="force the shape-generic kernels")
    ap.add_argument("--bf16-checkpoints", action="store_true", help="keep the segment checkpoints in bf16 (half the bytes)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-peak", action="store_true", help="skip the two passes that measure peak memory (profiler runs: every launch of the run then has the benchmark's shape)")
    ap.add_argument("--timed-only", action="store_true", help="profiler runs: warm-up and the timed steps only, no per-kernel passes")
    ap.add_argument("--no-extras", action="store_true", help="skip the L = 2^20 layer and the 16-layer stack (configs_extra)")
    ap.add_argument("--inference", action="store_true",
                    help="instead of the training step: forward-only prefill without checkpoints (tokens/s) and the "
                         "token-by-token recurrent step (us per token) at the same layer shape")
    ap.add_argument("--conv", action="store_true",
                    help="instead of the scan: the block's causal depthwise convolution + SiLU (forward and backward) at the "
                         "2.7B block's width, against the HBM roofline")
    ap.add_argument("--norm", action="store_true",
                    help="time the block's gated RMS normalisation (forward + backward) at the config's width instead")
    ap.add_argument("--linear", action="store_true",
                    help="time the block's input and output projections (forward, input and weight gradients) instead")
    ap.add_argument("--block", action="store_true",
                    help="time one whole Mamba-2 block (projections, convolution, scan, gated norm) under sequence checkpoints instead")
    ap.add_argument("--pre-norm", action="store_true", help="with --block: each block starts with an RMS normalisation of its input")
    ap.add_argument("--layers", type=int, default=1, help="with --block: a residual stack of this many blocks on the two-axis grid")
    ap.add_argument("--layer-interval", type=int, default=4, help="with --block --layers: layer inputs kept every this many layers")
    ap.add_argument("--calibrate-mfma", action="store_true",
                    help="run a register-only MFMA loop over the whole chip and print the rate it sustains")
    ap.add_argument("--calibrate-clock", action="store_true",
                    help="measure the shader clock while the projection GEMM, a register-only MFMA loop, a device copy and the scan run")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a device-to-device copy of 1 GiB, five times (reference for the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2411_19460_amd as pk
    from paper_2411_19460_amd import synth

    if args.calibrate_copy:
        torch.cuda.set_device(0)
        a = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0").normal_()
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(5):
            b.copy_(a)
        torch.cuda.synchronize()
        dtc = (time.perf_counter() - t0) / 5
        print(json.dumps({"copy_bytes_read": a.numel() * 4, "copy_bytes_written": a.numel() * 4, "copies": 5,
                          "GB_per_s_read_plus_write": 2 * a.numel() * 4 / dtc / 1e9}))
        return
    cfg = synth.CONFIGS[args.config]
    if args.segment:
        cfg = cfg.scaled(segment=args.segment)
    if cfg.nlayers != 1:
        print("bench.py: stack configs are measured by tests, not by this bench", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.calibrate_clock:
        # the shader clock while a kernel runs: a one-wave probe on a second stream counts shader cycles against
        # the constant 100 MHz counter for 30 ms while the work fills the first stream
        L = pk.lib()
        L.ssd_prof_clock_probe.argtypes = [ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p]
        L.ssd_prof_mfma_peak.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p]
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        out = torch.zeros(2, dtype=torch.int64, device=dev)
        T, I, O = 65536, 2560, 10576
        x = torch.randn(T, I, device=dev).to(torch.bfloat16)
        w = (torch.randn(O, I, device=dev) / 50).to(torch.bfloat16)
        y = torch.empty(T, O, dtype=torch.bfloat16, device=dev)
        sink = torch.zeros(1, device=dev)
        z = torch.empty(1 << 28, dtype=torch.float32, device=dev)
        z2 = torch.empty_like(z)
        d = synth.make_layer_inputs_device(cfg, dev)

        def scan_step():
            _, _, bs = pk.ssd_fwd(d["x"], d["dt"], d["A"], d["B"], d["C"], d["D"], cfg.chunk, cfg.segment)
            pk.ssd_bwd(d["x"], d["dt"], d["A"], d["B"], d["C"], d["D"], d["dy"], cfg.chunk, cfg.segment, boundary_states=bs)
        res = {}
        for label, work in (("idle", lambda: None),
                            ("input_projection_x12", lambda: [pk.ssd_linear_fwd(x, w, y) for _ in range(12)]),
                            ("mfma_on_registers", lambda: L.ssd_prof_mfma_peak(30000, 1024, sink.data_ptr(), torch.cuda.current_stream().cuda_stream)),
                            ("device_copy_1GiB_x40", lambda: [z2.copy_(z) for _ in range(40)]),
                            ("ssd_fwd_bwd_x8", lambda: [scan_step() for _ in range(8)])):
            with torch.cuda.stream(s1):
                work()   # warm
            torch.cuda.synchronize()
            assert L.ssd_prof_clock_probe(3000000, out.data_ptr(), s2.cuda_stream) == 0
            t0 = time.perf_counter()
            with torch.cuda.stream(s1):
                work()
            s1.synchronize()
            ms = (time.perf_counter() - t0) * 1e3
            torch.cuda.synchronize()
            wt, cy = out.tolist()
            res[label] = {"work_ms": ms, "probe_ms": wt / 1e5, "shader_clock_GHz": cy / (wt / 100.0) / 1e3}
        print(json.dumps({"calibration": "shader clock beside the work (30 ms probe)", **res}))
        return
    if args.calibrate_mfma:
        # sustained rate of the matrix cores on registers only: 1024 workgroups (four per compute unit in turn)
        sink = torch.zeros(1, device=dev)
        iters, wgs = 20000, 1024
        out = {}
        for label, n in (("short", 2000), ("long", iters)):
            for _ in range(2):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                rc = pk.lib().ssd_prof_mfma_peak(n, wgs, sink.data_ptr(), torch.cuda.current_stream().cuda_stream or None)
                e1.record()
                torch.cuda.synchronize()
                assert rc == 0
            ms = e0.elapsed_time(e1)
            out[label] = {"ms": ms, "TFLOP/s": wgs * 4 * n * 16 * 32768.0 / (ms * 1e-3) / 1e12}
        print(json.dumps({"calibration": "mfma_f32_32x32x16_bf16 on registers", "nominal_peak_TFLOP/s": MFMA_BF16_PEAK_TFLOPS, **out}))
        return
    if args.block:
        block_bench(args, cfg, pk, torch, dev)
        return
    if args.inference:
        inference_bench(args, cfg, pk, synth, torch, dev)
        return
    if args.conv:
        conv_bench(args, cfg, pk, torch, dev)
        return
    if args.norm:
        norm_bench(args, cfg, pk, torch, dev)
        return
    if args.linear:
        linear_bench(args, cfg, pk, torch, dev)
        return
    if args.block:
        block_bench(args, cfg, pk, torch, dev)
        return
    flags = pk.SSD_FLAG_GENERIC_KERNELS if args.generic else 0
    if args.bf16_checkpoints:
        flags |= pk.SSD_FLAG_BF16_CHECKPOINTS
    Bt, L, H, P, N, G = cfg.batch, cfg.seqlen, cfg.nheads, cfg.headdim, cfg.dstate, cfg.ngroups
    main = layer_bench(cfg, args.steps, args.warmup, flags, pk, synth, torch, dev, per_kernel=not args.timed_only,
                       measure_peak=not args.no_peak)
    if args.timed_only:   # profiler runs that want nothing but launches of the timed configuration
        print(json.dumps({"metric": "SSD fwd+bwd tokens/sec/layer", "value": main["tokens_per_s"], "unit": "tokens/s",
                          "ms_per_step": main["ms_per_step"], "median_ms_per_step": main["median_ms_per_step"],
                          "config": {"workload": cfg.name}, "note": "timed region only (no per-kernel pass, no roofline)"}))
        return
    tok_s, ms_per_step = main["tokens_per_s"], main["ms_per_step"]
    kernels, dom = main["kernels_serialized"], main["dominant"]
    group = KERNEL_GROUP.get(dom, "bwd")
    gbytes = group_bytes(cfg)[group] * Bt * cfg.segment      # algorithmic bytes of the kernel's group per launch (one segment)
    dsec = kernels[dom]["avg_us"] * 1e-6
    roofline = {"kernel": dom, "bound": "hbm", "achieved": gbytes / dsec / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": gbytes / dsec / 1e9 / HBM_PEAK_GBS, "traffic": measured_traffic(dom, cfg.name),
                "algorithmic_bytes_per_launch": gbytes, "avg_launch_us": kernels[dom]["avg_us"],
                "duration": "kernel alone on the GPU (every segment on one stream), HIP events around each launch, "
                            "untimed pass after the timed region",
                "bytes": f"{group} group of the path per token ({group_bytes(cfg)[group]:.0f} B: inputs read once, outputs "
                         f"written once) x {Bt * cfg.segment} tokens per launch",
                "in_flight_avg_launch_us": main["dominant_in_flight_us"],
                "share_of_kernel_time": kernels[dom]["ms_per_step"] / sum(k["ms_per_step"] for k in kernels.values()),
                "tflops": kernels[dom].get("tflops"), "frac_mfma": (kernels[dom].get("tflops") or 0.0) / MFMA_BF16_PEAK_TFLOPS}
    pfl, pby = path_model(cfg)
    roofline_path = {"bound": "hbm" if pfl / pby < MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9) else "mfma",
                     "algorithmic_bytes_per_token": pby, "algorithmic_flop_per_token": pfl,
                     "achieved_gbs": pby * tok_s / 1e9, "frac_hbm": pby * tok_s / 1e9 / HBM_PEAK_GBS,
                     "achieved_tflops": pfl * tok_s / 1e12, "frac_mfma": pfl * tok_s / 1e12 / MFMA_BF16_PEAK_TFLOPS}
    res = {
        "metric": "SSD fwd+bwd tokens/sec/layer", "value": tok_s, "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "batch": Bt, "seqlen": L, "nheads": H, "headdim": P, "dstate": N,
                   "ngroups": G, "chunk": cfg.chunk, "segment": cfg.segment,
                   "checkpoints": "bf16" if args.bf16_checkpoints else "f32",
                   "kernels": "generic" if args.generic or not any(k.startswith("mfma_") for k in kernels) else "mfma",
                   "segments_in_flight": min(4, L // cfg.segment) if not args.generic else 1},
        "median_ms_per_step": main["median_ms_per_step"], "step_ms": main["step_ms"],
        "roofline": roofline, "roofline_path": roofline_path, "kernels_serialized": kernels, "peak_hbm": main["peak_hbm"],
    }
    if not args.no_extras and args.config == 2 and not args.segment and not args.generic:
        del main
        torch.cuda.empty_cache()
        extra = {}
        c3 = synth.CONFIGS[3]
        r3 = layer_bench(c3, 3, 1, flags, pk, synth, torch, dev, per_kernel=False)
        extra[c3.name] = {"tokens_per_s": r3["tokens_per_s"], "ms_per_step": r3["ms_per_step"],
                          "median_ms_per_step": r3["median_ms_per_step"], "segment": c3.segment, "peak_hbm": r3["peak_hbm"]}
        del r3
        torch.cuda.empty_cache()
        extra[synth.CONFIGS[4].name] = stack_bench(synth.CONFIGS[4], 2, 1, pk, synth, torch, dev)
        res["configs_extra"] = extra
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
