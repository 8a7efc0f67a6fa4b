"""GPU parity of the block's projections (forward, input gradient, weight gradient) against the fp64
oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2411_19460_amd as pk
from oracle import linear_ref
from paper_2411_19460_amd import synth
from parity_util import TOL, check, host

pytestmark = pytest.mark.gpu


def draw(seed, T, I, O):
    r = np.random.default_rng(3000 + seed)
    f = lambda a: np.asarray(synth.round_bf16(a), dtype=np.float64)
    return f(r.standard_normal((T, I))), f(r.standard_normal((O, I)) / np.sqrt(I)), f(r.standard_normal((T, O)))


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda().to(torch.bfloat16)


def in_wider(t, width, col0):
    wide = torch.zeros((t.shape[0], width), dtype=t.dtype, device=t.device)
    view = wide[:, col0:col0 + t.shape[1]]
    view.copy_(t)
    return view


@pytest.mark.parametrize("case", [
    # rows, in_dim, out_dim, operands as column slices of wider tensors
    (300, 64, 72, False),          # one K step, ragged tiles in both directions
    (513, 136, 200, False),        # K not a multiple of the K step
    (1000, 2560, 10576, False),    # the 2.7B block's input projection (d_model -> 2 d_inner + 2 G N + H), ragged rows
    (520, 5120, 2560, False),      # its output projection
    (260, 264, 136, True),         # x, out, dout, dx as slices (16-byte aligned, rows further apart)
    (5, 8, 8, False),              # smaller than any tile
])
def test_linear_forward_backward(case):
    T, I, O, sliced = case
    x, w, dout = draw(1, T, I, O)
    xd, wd, dd = dev(x), dev(w), dev(dout)
    if sliced:
        xd, dd = in_wider(xd, I + 24, 8), in_wider(dd, O + 40, 16)
    out = in_wider(torch.zeros((T, O), dtype=torch.bfloat16, device="cuda"), O + 16, 8) if sliced else None
    out = pk.ssd_linear_fwd(xd, wd, out)
    tol = TOL["bf16"]
    check("out", host(out), linear_ref.linear_fwd(x, w), tol)
    dx = in_wider(torch.zeros((T, I), dtype=torch.bfloat16, device="cuda"), I + 8, 0) if sliced else None
    g = pk.ssd_linear_bwd(xd, wd, dd, dx=dx)
    torch.cuda.synchronize()
    ref = linear_ref.linear_bwd(x, w, dout)
    rep = {}
    check("dx", host(g["dx"]), ref["dx"], tol, rep)
    check("dw", host(g["dw"]), ref["dw"], 1e-4, rep)           # fp32 sums of exact bf16 products
    print("linear errors:", {k: f"{v:.2e}" for k, v in rep.items()})
    if sliced:   # nothing outside the slices was written
        for view, c0, n in ((out, 8, O), (g["dx"], 0, I)):
            wide = view._base
            mask = torch.ones(wide.shape, dtype=torch.bool, device=wide.device)
            mask[:, c0:c0 + n] = False
            assert float(wide[mask].float().abs().max()) == 0.0
    g2 = pk.ssd_linear_bwd(xd, wd, dd, want_dx=False, flags=pk.SSD_FLAG_ACCUM_PARAM, dw=g["dw"].clone())
    assert g2["dx"] is None
    check("dw accumulated", host(g2["dw"]), 2 * ref["dw"], 1e-4)


@pytest.mark.parametrize("case", [(1, 2560, 10576, False), (1, 5120, 2560, False), (3, 136, 200, True), (16, 520, 72, True), (7, 8, 8, False)])
def test_linear_forward_for_a_few_rows(case):
    """A token or a few (generation): the product that reads the weights once, one wave per pair of columns."""
    T, I, O, sliced = case
    x, w, _ = draw(2, T, I, O)
    xd, wd = dev(x), dev(w)
    out = None
    if sliced:
        xd = in_wider(xd, I + 24, 8)
        out = in_wider(torch.zeros((T, O), dtype=torch.bfloat16, device="cuda"), O + 16, 8)
    out = pk.ssd_linear_fwd(xd, wd, out)
    torch.cuda.synchronize()
    check("out", host(out), linear_ref.linear_fwd(x, w), TOL["bf16"])
    if sliced:
        wide = out._base
        mask = torch.ones(wide.shape, dtype=torch.bool, device=wide.device)
        mask[:, 8:8 + O] = False
        assert float(wide[mask].float().abs().max()) == 0.0


def test_linear_empty_and_rejected_arguments():
    x = torch.zeros((0, 64), dtype=torch.bfloat16, device="cuda")
    w = torch.ones((16, 64), dtype=torch.bfloat16, device="cuda")
    assert pk.ssd_linear_fwd(x, w).shape == (0, 16)
    g = pk.ssd_linear_bwd(x, w, torch.zeros((0, 16), dtype=torch.bfloat16, device="cuda"))
    torch.cuda.synchronize()
    assert float(g["dw"].abs().max()) == 0.0
    with pytest.raises(pk.SSDError):
        pk.ssd_linear_fwd(torch.zeros((4, 12), dtype=torch.bfloat16, device="cuda"),
                          torch.zeros((8, 12), dtype=torch.bfloat16, device="cuda"))      # 12 is not a multiple of 8
    wide = torch.zeros((4, 80), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(pk.SSDError):
        pk.ssd_linear_fwd(wide[:, 4:68], w)                                               # slice not 16-byte aligned
