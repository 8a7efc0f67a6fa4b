"""Helpers shared by the GPU parity tests: move seeded inputs to the device, run the HIP path
through the C ABI, run the fp64 oracle on the same (already rounded) values, compare."""
import numpy as np
import torch

import paper_2411_19460_amd as pk
from oracle import ssd_ref

TOL = {"f32": 1e-3, "bf16": 2e-2}   # max |gpu - ref| / max |ref| per tensor


def to_dev(a, dtype):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def dev_inputs(d, dtype):
    out = {}
    for k, v in d.items():
        if v is None:
            out[k] = None
        elif k in ("A", "D", "init_state", "dfinal_state"):
            out[k] = torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32)).cuda()
        else:
            out[k] = to_dev(v, dtype)
    return out


def host(t):
    return None if t is None else t.detach().float().cpu().numpy().astype(np.float64)


def rel_err(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    scale = float(np.max(np.abs(ref))) if ref.size else 0.0
    if ref.size == 0:
        return 0.0
    return float(np.max(np.abs(np.asarray(got, dtype=np.float64) - ref))) / (scale if scale > 0 else 1.0)


def check(name, got, ref, tol, report=None):
    assert np.all(np.isfinite(got)), f"{name}: non-finite values"
    e = rel_err(got, ref)
    if report is not None:
        report[name] = e
    assert e <= tol, f"{name}: max-normalised error {e:.3e} > {tol:.1e}"


def run_gpu(dv, chunk, segment, flags=0):
    y, fin, bnd = pk.ssd_fwd(dv["x"], dv["dt"], dv["A"], dv["B"], dv["C"], dv["D"], chunk, segment,
                             dv.get("init_state"), flags)
    g = pk.ssd_bwd(dv["x"], dv["dt"], dv["A"], dv["B"], dv["C"], dv["D"], dv["dy"], chunk, segment,
                   dv.get("init_state"), dv.get("dfinal_state"), bnd, flags)
    torch.cuda.synchronize()
    return y, fin, bnd, g


def run_oracle(d, segment=None, head_group=None):
    f = ssd_ref.ssd_fwd(d["x"], d["dt"], d["A"], d["B"], d["C"], d["D"], d.get("init_state"), segment, head_group)
    g = ssd_ref.ssd_bwd(d["x"], d["dt"], d["A"], d["B"], d["C"], d["D"], d["dy"], d.get("init_state"),
                        d.get("dfinal_state"), head_group)
    return f, g


def compare_all(d, dtype, chunk, segment, flags=0, residual=False, report=None):
    """Full element-by-element comparison of every output with the oracle."""
    dv = dev_inputs(d, dtype)
    y, fin, bnd, g = run_gpu(dv, chunk, segment, flags)
    f, go = run_oracle(d, segment)
    tol = TOL[dtype]
    yref = f["y"] + (d["x"] if residual else 0.0)
    check("y", host(y), yref, tol, report)
    check("final_state", host(fin), f["final_state"], tol, report)
    if segment is not None:
        check("boundary_states", host(bnd), f["boundary_states"], tol, report)
    dxref = go["dx"] + (d["dy"] if residual else 0.0)
    check("dx", host(g["dx"]), dxref, tol, report)
    for k in ("ddt", "dA", "dB", "dC", "dD", "dinit_state"):
        check(k, host(g[k]), go[k], tol, report)
    return dv, (y, fin, bnd, g)
