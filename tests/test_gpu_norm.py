"""GPU parity of the block's gated RMS normalisation (forward and backward) against the fp64 oracle,
through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2411_19460_amd as pk
from oracle import norm_ref
from paper_2411_19460_amd import synth
from parity_util import TOL, check, host

pytestmark = pytest.mark.gpu


def draw(seed, dtype, T, C):
    r = np.random.default_rng(2000 + seed)
    rnd = synth.round_bf16 if dtype == "bf16" else (lambda a: a.astype(np.float32))
    f = lambda a: np.asarray(rnd(a), dtype=np.float64)
    return dict(y=f(r.standard_normal((T, C))), z=f(2.0 * r.standard_normal((T, C))),
                w=(1.0 + 0.3 * r.standard_normal(C)).astype(np.float32).astype(np.float64), dout=f(r.standard_normal((T, C))))


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def in_wider(t, width, col0):
    """The same values as a column slice [:, col0:col0+C] of a [T, width] tensor (rows `width` apart)."""
    wide = torch.zeros((t.shape[0], width), dtype=t.dtype, device=t.device)
    view = wide[:, col0:col0 + t.shape[1]]
    view.copy_(t)
    return view


@pytest.mark.parametrize("case", [
    # dtype, rows, dim, groups, z as a slice of a tensor this wide (0 = dense), first column of the slice
    ("bf16", 1000, 5120, 1, 0, 0),        # the 2.7B block (d_inner), rows not a multiple of the tile
    ("bf16", 300, 5120, 8, 10576, 0),     # eight groups; z is the leading slice of the input projection's output
    ("bf16", 64, 16384, 1, 0, 0),         # the widest segment the register-resident kernel takes
    ("bf16", 70, 16392, 1, 0, 0),         # wider: element-wise kernel
    ("bf16", 65, 1032, 1, 2048, 3),       # slice that starts at an odd column: not 16-byte aligned
    ("f32", 130, 96, 3, 0, 0),
    ("f32", 70, 30, 2, 0, 0),             # group size not a multiple of the vector width
    ("f32", 3, 2048, 1, 0, 0),            # fewer rows than waves in a tile
])
def test_gated_norm_forward_backward(case):
    dtype, T, C, G, width, col0 = case
    d = draw(1, dtype, T, C)
    y, z, dout = (dev(d[k], dtype) for k in ("y", "z", "dout"))
    w = dev(d["w"])
    if width:
        z = in_wider(z, width, col0)
    tol = TOL[dtype]
    out = pk.ssd_gated_norm_fwd(y, z, w, 1e-5, G)
    check("out", host(out), norm_ref.gated_rmsnorm_fwd(d["y"], d["z"], d["w"], 1e-5, G), tol)
    dz = in_wider(torch.zeros_like(y), width, col0) if width else None
    g = pk.ssd_gated_norm_bwd(y, z, w, dout, 1e-5, G, dz=dz)
    torch.cuda.synchronize()
    ref = norm_ref.gated_rmsnorm_bwd(d["y"], d["z"], d["w"], d["dout"], 1e-5, G)
    rep = {}
    for k in ("dy", "dz", "dw"):
        check(k, host(g[k]), ref[k], tol, rep)
    print("gated norm errors:", {k: f"{v:.2e}" for k, v in rep.items()})
    if width:   # nothing outside the slice was touched
        wide = dz._base if dz._base is not None else dz
        mask = torch.ones(wide.shape, dtype=torch.bool, device=wide.device)
        mask[:, col0:col0 + C] = False
        assert float(wide[mask].float().abs().max()) == 0.0
    # accumulation into dw
    g2 = pk.ssd_gated_norm_bwd(y, z, w, dout, 1e-5, G, flags=pk.SSD_FLAG_ACCUM_PARAM, dw=g["dw"].clone())
    check("dw accumulated", host(g2["dw"]), 2 * ref["dw"], tol)


@pytest.mark.parametrize("case", [("bf16", 1000, 2560, 1), ("bf16", 37, 16392, 1), ("f32", 130, 96, 3)])
def test_norm_without_a_gate(case):
    """z == NULL: the plain RMS normalisation (a block's pre-norm at the 2.7B model width, the element-wise
    kernel, fp32 with groups)."""
    dtype, T, C, G = case
    d = draw(5, dtype, T, C)
    y, dout = dev(d["y"], dtype), dev(d["dout"], dtype)
    w = dev(d["w"])
    tol = TOL[dtype]
    check("out", host(pk.ssd_gated_norm_fwd(y, None, w, 1e-5, G)), norm_ref.gated_rmsnorm_fwd(d["y"], None, d["w"], 1e-5, G), tol)
    g = pk.ssd_gated_norm_bwd(y, None, w, dout, 1e-5, G)
    torch.cuda.synchronize()
    ref = norm_ref.gated_rmsnorm_bwd(d["y"], None, d["w"], d["dout"], 1e-5, G)
    assert g["dz"] is None
    for k in ("dy", "dw"):
        check(k, host(g[k]), ref[k], tol)


def test_gated_norm_empty_and_rejected_arguments():
    y = torch.zeros((0, 64), dtype=torch.bfloat16, device="cuda")
    w = torch.ones(64, device="cuda")
    assert pk.ssd_gated_norm_fwd(y, y, w).shape == (0, 64)
    g = pk.ssd_gated_norm_bwd(y, y, w, y)
    torch.cuda.synchronize()
    assert float(g["dw"].abs().max()) == 0.0
    y = torch.zeros((4, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(pk.SSDError):
        pk.ssd_gated_norm_fwd(y, y, w, 1e-5, 5)       # 64 channels do not split into 5 groups
    with pytest.raises(pk.SSDError):
        pk.ssd_gated_norm_fwd(y, y, w, -1.0, 1)       # negative eps
