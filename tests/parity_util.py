"""Helpers shared by the GPU parity tests: move seeded inputs to the device, run the HIP path
through the C ABI, run the fp64 oracle on the same (already rounded) values, compare."""
import numpy as np
import torch

import paper_2411_19460_amd as pk
from oracle import ssd_ref

TOL = {"f32": 1e-3, "bf16": 2e-2}   # max |gpu - ref| / max |ref| per tensor


def stack_tol(dtype, nlayers):
    """Tolerance for the output of a residual stack of `nlayers` layers.  TOL is the bar for one layer.  A layer
    adds its own error (measured: 3-5e-3 of the largest magnitude in bf16, a quarter of TOL) to a residual stream
    that carries the errors of the layers below with the same gain as the signal, so the error after n layers grows
    like that of a random walk, sqrt(n) times the single-layer error: with the single layer allowed TOL / 2 of
    head room before the stack is, the bar is TOL * sqrt(n) / 2, never below TOL (n = 16: 2 TOL)."""
    return TOL[dtype] * max(1.0, nlayers ** 0.5 / 2.0)


def check_dot_gradient(name, got, ref, a, b, tol, report=None):
    """A gradient that is a plain dot product sum_i a_i b_i of two stored tensors (dD = sum dy x): when the
    two are nearly uncorrelated the sum is the small remainder of a large cancellation, and rounding each factor
    once (relative error delta) already moves it by delta * sqrt(sum_i (a_i b_i)^2), however small the sum itself
    is.  The error is therefore measured against max(|ref|, sqrt(sum_i (a_i b_i)^2)): a missing or misplaced
    part of the sum changes it by a multiple of that scale, a rounding order does not."""
    scale = max(abs(float(ref)), float(np.sqrt(np.sum((np.asarray(a, dtype=np.float64) * np.asarray(b, dtype=np.float64)) ** 2))))
    e = abs(float(got) - float(ref)) / (scale if scale > 0 else 1.0)
    if report is not None:
        report[name] = max(report.get(name, 0.0), e)
    assert np.isfinite(e) and e <= tol, f"{name}: |gpu - ref| / scale = {e:.3e} > {tol:.1e} (gpu {float(got):.4g}, ref {float(ref):.4g})"


def progress(text):
    """A step of a long test is done: one line into gpurun_out/pytest_progress.log under the repository root when
    that folder exists (where a runner that watches for output looks while pytest holds stdout back), else nothing."""
    import os
    folder = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "gpurun_out")
    if os.path.isdir(folder):
        with open(os.path.join(folder, "pytest_progress.log"), "a") as f:
            f.write(text + "\n")


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
