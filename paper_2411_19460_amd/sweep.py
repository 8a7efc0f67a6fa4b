#!/usr/bin/env python3
"""Memory and time of a residual stack of SSD layers against the sequence length, for three
checkpoint grids (Sec. 3.2-3.3, Alg. 1-2; the experiment of Tab. 3 / Fig. 1 at SSD-layer scale):

  per-layer : every layer input is kept for the whole sequence (l = 1, s = S): O(L S) memory
  sqrt-L    : every sqrt(L)-th layer input is kept (s = S)
  MA-GC     : the two-axis grid (l, s) that `magc_plan` picks for this S: O(S) memory with a small slope

    python -m paper_2411_19460_amd.sweep [--layers 16] [--min-log2 12] [--max-log2 20] [--budget-gb 200]

Prints one JSON line per (S, grid) and a table at the end.  Inputs are seeded synthetic tensors at the
2.7B layer shape; configurations whose checkpoints + workspace exceed the budget are reported as
predicted only (sizes come from the library's own workspace queries, which are exact).
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--layers", type=int, default=16)
    ap.add_argument("--min-log2", type=int, default=12)
    ap.add_argument("--max-log2", type=int, default=20)
    ap.add_argument("--step-log2", type=int, default=2)
    ap.add_argument("--budget-gb", type=float, default=200.0)
    ap.add_argument("--pareto", default="", help="with --blocks: comma-separated memory budgets in GB; runs the planner's budget mode for each instead of the three grids")
    ap.add_argument("--pre-norm", action="store_true", help="with --blocks: every block starts with an RMS normalisation of its input")
    ap.add_argument("--blocks", action="store_true",
                    help="whole Mamba-2 blocks (projections, convolution, scan, gated norm) instead of bare SSD layers")
    args = ap.parse_args()
    if args.blocks:
        return blocks_sweep(args)

    import torch
    import paper_2411_19460_amd as pk
    from paper_2411_19460_amd import synth

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    base = synth.CONFIGS[4]
    H, P, N, G, Q, nl = base.nheads, base.headdim, base.dstate, base.ngroups, base.chunk, args.layers
    # per-token / per-checkpoint sizes of this implementation, in bytes (bf16 activations, fp32 checkpointed states,
    # bf16 chunk states and adjoints of the layer being processed)
    c_l, c_s, c_grid, c_state = H * P * 2, H * P * N * 4, H * P * 2, 2 * H * P * N * 2 // Q
    rows = []
    for lg in range(args.min_log2, args.max_log2 + 1, args.step_log2):
        S = 1 << lg
        rc, plan = pk.magc_plan(nl, S, c_l, c_s, c_grid, c_state, s_multiple=Q, integer_counts=True)
        # the kernels need S to be a whole number of segments: take the power of two next to the planned interval
        s_plan = min(S, max(Q, 1 << int(round(math.log2(plan["s"])))))
        grids = [("per-layer", 1, S), ("sqrt-L", max(1, int(round(math.sqrt(nl)))), S), ("MA-GC", plan["l"], s_plan)]
        cfg = base.scaled(seqlen=S, nlayers=nl, name=f"stack{nl}_2^{lg}")
        data = None
        for name, l, s in grids:
            shape = pk.ssd_shape_t(pk.SSD_BF16, H, P, G, N, Q, 1, S, s, 0, 0, 0)
            nlg = (nl + l - 1) // l
            ckpt = nl * (S // s) * c_s + (nlg - 1) * S * c_l
            ws = max(pk.magc_stack_workspace_bytes(shape, nl, l, False), pk.magc_stack_workspace_bytes(shape, nl, l, True))
            row = {"S": S, "grid": name, "l": l, "s": s, "s_planned": plan["s"] if name == "MA-GC" else None, "checkpoint_bytes": ckpt, "workspace_bytes": ws,
                   "kept_bytes": ckpt + ws, "ran": False}
            if (ckpt + ws) / 1e9 <= args.budget_gb:
                if data is None:
                    layers = []
                    for j in range(nl):   # x of the deeper layers is not an input: drop it at once
                        lay = synth.make_layer_inputs_device(cfg, dev, layer=j, with_dy=(j == 0))
                        if j == 0:
                            x0, dout = lay["x"], lay["dy"]
                        layers.append({k: lay[k] for k in ("dt", "A", "B", "C", "D")})
                        del lay
                    data = {k: torch.stack([lay[k] for lay in layers]).contiguous() for k in ("dt", "A", "B", "C", "D")}
                    del layers
                a = [data[k] for k in ("dt", "A", "B", "C", "D")]

                def step():
                    f = pk.magc_stack_fwd(x0, *a, Q, s, l, want_final=False)
                    b = pk.magc_stack_bwd(x0, *a, dout, f["s_ckpt"], f["l_ckpt"], Q, s, l)
                    return f, b

                # pass 1, from an empty allocator cache: the memory figures
                torch.cuda.synchronize()
                torch.cuda.empty_cache()
                base_mem = torch.cuda.memory_allocated()
                torch.cuda.reset_peak_memory_stats()
                f, b = step()
                torch.cuda.synchronize()
                peak = torch.cuda.max_memory_allocated() - base_mem
                ok = bool(torch.isfinite(b["dx0"].float().sum()))
                del f, b
                # pass 2, allocator warm (no device allocation inside the timed region): the time
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                f, b = step()
                torch.cuda.synchronize()
                ms = (time.perf_counter() - t0) * 1e3
                del f, b
                row.update({"ran": True, "ms": ms, "tokens_per_s_per_layer": nl * S / (ms * 1e-3),
                            "peak_beyond_inputs_bytes": peak, "finite": ok})
            print(json.dumps(row), flush=True)
            rows.append(row)
        del data
        torch.cuda.empty_cache()
    print("\n| S | grid | l | s | checkpoints + workspace | peak beyond inputs (incl. outputs) | ms fwd+bwd | M tok/s/layer |")
    print("|---|---|---|---|---|---|---|---|")
    for r in rows:
        kept = f"{r['kept_bytes'] / 1e9:.2f} GB"
        if r["ran"]:
            print(f"| 2^{int(math.log2(r['S']))} | {r['grid']} | {r['l']} | {r['s']} | {kept} | "
                  f"{r['peak_beyond_inputs_bytes'] / 1e9:.2f} GB | {r['ms']:.1f} | {r['tokens_per_s_per_layer'] / 1e6:.2f} |")
        else:
            print(f"| 2^{int(math.log2(r['S']))} | {r['grid']} | {r['l']} | {r['s']} | {kept} (predicted, over budget) | - | - | - |")


def blocks_sweep(args):
    """The same experiment with whole blocks at the 2.7B widths (d_model 2560): a residual stack of --layers
    blocks, forward + backward, on the three grids.  Closest to the paper's own table: its model is such a stack."""
    import ctypes

    import torch
    import paper_2411_19460_amd as pk
    from paper_2411_19460_amd import binding, synth

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    base = synth.CONFIGS[2]
    H, P, N, G, Q, nl = base.nheads, base.headdim, base.dstate, base.ngroups, base.chunk, args.layers
    d_inner, dm = H * P, H * P // 2
    gn = G * N
    conv_dim, d_in_proj = d_inner + 2 * gn, 2 * d_inner + 2 * gn + H
    g = torch.Generator(device=dev)
    g.manual_seed(base.seed(0) + 23)
    rn = lambda *s: torch.randn(s, device=dev, generator=g, dtype=torch.float32)

    def layer():
        dt0 = torch.exp(torch.empty(H, device=dev).uniform_(math.log(1e-3), math.log(0.1), generator=g))
        return {"W_in": (rn(d_in_proj, dm) / dm ** 0.5).to(torch.bfloat16), "conv_w": rn(conv_dim, 4) * 0.5, "conv_b": rn(conv_dim) * 0.2,
                "dt_bias": dt0 + torch.log(-torch.expm1(-dt0)),
                "A": -torch.exp(torch.empty(H, device=dev).uniform_(0.0, math.log(16.0), generator=g)), "D": rn(H),
                "norm_w": 1.0 + 0.3 * rn(d_inner), "W_out": (rn(dm, d_inner) / d_inner ** 0.5 / nl ** 0.5).to(torch.bfloat16),
                **({"pre_norm_w": 1.0 + 0.3 * rn(dm)} if args.pre_norm else {})}

    layers = [layer() for _ in range(nl)]
    grads = [{"d" + k: torch.empty(v.shape, dtype=torch.float32, device=dev) for k, v in layers[0].items()} for _ in range(nl)]

    def sshape(S, s, l):
        return binding.magc_blockstack_shape_t(binding.magc_block_shape_t(dm, H, P, G, N, Q, 1e-5, S, s), nl, l)

    # per-token / per-checkpoint sizes of this implementation in bytes: a kept layer input; both states of a layer;
    # what a cell keeps per layer and token (layer input, zxbcdt, y); the scratch of the layer being processed
    c_l, c_s, c_grid = dm * 2, H * P * N * 4 + 3 * conv_dim * 2, (dm + d_in_proj + d_inner) * 2
    seg = binding.magc_block_shape_t(dm, H, P, G, N, Q, 1e-5, 4096, 4096)
    c_state = int(pk.lib().magc_block_workspace_bytes(ctypes.byref(seg), 1)) // 4096
    rows = []
    for lg in range(args.min_log2, args.max_log2 + 1, args.step_log2):
        S = 1 << lg
        rc, plan = pk.magc_plan(nl, S, c_l, c_s, c_grid, c_state, s_multiple=Q, integer_counts=True)
        s_plan = min(S, max(Q, 1 << int(round(math.log2(plan["s"])))))
        grids = [("per-layer", 1, S), ("sqrt-L", max(1, int(round(math.sqrt(nl)))), S), ("MA-GC", plan["l"], s_plan)]
        if args.pareto:
            # the planner's other mode: for each memory budget the grid with the least recomputation that fits
            # (largest s, then largest l) -- the time / memory trade-off between the minimum-memory grid and no
            # sequence checkpoints at all
            grids = [("MA-GC min", plan["l"], plan["s"])]
            for gb in (float(v) for v in args.pareto.split(",")):
                rcb, pb = pk.magc_plan(nl, S, c_l, c_s, c_grid, c_state, s_multiple=Q, budget=gb * 1e9, integer_counts=True)
                if rcb == 0:
                    grids.append((f"budget {gb:g} GB", pb["l"], pb["s"]))
        # for scale: no checkpointing at all would keep, per layer and token, everything its backward reads -- the layer
        # input, zxbcdt, the activated xBC, dt, y and the normalised y (not run: the library always recomputes)
        c_all = (dm + d_in_proj + conv_dim + H + 2 * d_inner) * 2
        rows.append({"S": S, "grid": "none", "l": 0, "s": S, "kept_bytes": nl * S * c_all, "ran": False, "predicted_only": True})
        x0 = dout = None
        for name, l, s in grids:
            sh = sshape(S, s, l)
            ngl = (nl + l - 1) // l
            ckpt = nl * -(-S // s) * c_s + (ngl - 1) * S * c_l
            ws = max(int(pk.lib().magc_blockstack_workspace_bytes(ctypes.byref(sh), 0)), int(pk.lib().magc_blockstack_workspace_bytes(ctypes.byref(sh), 1)))
            row = {"S": S, "grid": name, "l": l, "s": s, "s_planned": plan["s"] if name == "MA-GC" else None, "checkpoint_bytes": ckpt,
                   "workspace_bytes": ws, "kept_bytes": ckpt + ws, "ran": False}
            if (ckpt + ws) / 1e9 <= args.budget_gb:
                if x0 is None:
                    x0, dout = rn(S, dm).to(torch.bfloat16), rn(S, dm).to(torch.bfloat16)

                def step():
                    f = pk.magc_blockstack_fwd(x0, layers, H, P, G, N, Q, s, l)
                    b = pk.magc_blockstack_bwd(x0, layers, dout, f["l_ckpt"], f["ssm_ckpt"], f["conv_ckpt"], H, P, G, N, Q, s, l, grads=grads)
                    return f, b

                torch.cuda.synchronize()
                torch.cuda.empty_cache()
                base_mem = torch.cuda.memory_allocated()
                torch.cuda.reset_peak_memory_stats()
                f, b = step()
                torch.cuda.synchronize()
                peak = torch.cuda.max_memory_allocated() - base_mem
                ok = bool(torch.isfinite(b["dx0"].float().sum())) and bool(torch.isfinite(grads[0]["dW_in"].sum()))
                del f, b
                print(f"# 2^{lg} {name}: memory pass done, peak {peak / 1e9:.2f} GB", flush=True)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                f, b = step()
                torch.cuda.synchronize()
                ms = (time.perf_counter() - t0) * 1e3
                del f, b
                row.update({"ran": True, "ms": ms, "tokens_per_s_per_layer": nl * S / (ms * 1e-3), "peak_beyond_inputs_bytes": peak, "finite": ok})
            print(json.dumps(row), flush=True)
            rows.append(row)
        del x0, dout
        torch.cuda.empty_cache()
    print("\n| S | grid | l | s | checkpoints + workspace | peak beyond inputs (incl. outputs) | s fwd+bwd | M tok/s/layer |")
    print("|---|---|---|---|---|---|---|---|")
    for r in rows:
        kept = f"{r['kept_bytes'] / 1e9:.2f} GB"
        if r["ran"]:
            print(f"| 2^{int(math.log2(r['S']))} | {r['grid']} | {r['l']} | {r['s']} | {kept} | "
                  f"{r['peak_beyond_inputs_bytes'] / 1e9:.2f} GB | {r['ms'] / 1e3:.2f} | {r['tokens_per_s_per_layer'] / 1e6:.2f} |")
        elif r.get("predicted_only"):
            print(f"| 2^{int(math.log2(r['S']))} | no checkpointing | - | - | {kept} (every activation kept; not run) | - | - | - |")
        else:
            print(f"| 2^{int(math.log2(r['S']))} | {r['grid']} | {r['l']} | {r['s']} | {kept} (predicted, over budget) | - | - | - |")


if __name__ == "__main__":
    main()
