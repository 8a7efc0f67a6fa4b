"""GPU parity of the residual stack on the MA-GC grid (layer and sequence checkpoints) against the
fp64 oracle, and invariance of the results under the choice of grid."""
import numpy as np
import pytest
import torch

import paper_2411_19460_amd as pk
from oracle import ssd_ref
from paper_2411_19460_amd import synth
from parity_util import TOL, check, host, stack_tol, to_dev

pytestmark = pytest.mark.gpu


def stack_inputs(cfg):
    layers = [synth.make_layer_inputs(cfg, layer=j) for j in range(cfg.nlayers)]
    x0, dout = layers[0]["x"], layers[0]["dy"]
    return x0, dout, layers


def stacked(layers, key, dtype):
    a = np.stack([l[key] for l in layers])
    if key in ("A", "D"):
        return torch.from_numpy(a.astype(np.float32)).cuda()
    return to_dev(a, dtype)


def run_stack(cfg, x0, dout, layers, l_int, seg):
    dt = cfg.dtype
    args = [stacked(layers, k, dt) for k in ("dt", "A", "B", "C", "D")]
    xd, dd = to_dev(x0, dt), to_dev(dout, dt)
    f = pk.magc_stack_fwd(xd, *args, cfg.chunk, seg, l_int)
    b = pk.magc_stack_bwd(xd, *args, dd, f["s_ckpt"], f["l_ckpt"], cfg.chunk, seg, l_int)
    torch.cuda.synchronize()
    return f, b


@pytest.mark.parametrize("dtype,l_int,seg", [("f32", 2, 64), ("f32", 5, 128), ("f32", 1, 256), ("bf16", 3, 128)])
def test_stack_matches_oracle(dtype, l_int, seg):
    cfg = synth.SSDConfig("stack", dtype, 1, 256, 3, 16, 16, 1, 32, seg, nlayers=5, index=60)
    x0, dout, layers = stack_inputs(cfg)
    # keep the residual stream O(1): D ~ N(0,1) would otherwise amplify it layer after layer
    f, b = run_stack(cfg, x0, dout, layers, l_int, seg)
    # the stack's activations and their gradients are tensors of the storage dtype: rounded once where stored
    store = synth.round_bf16 if dtype == "bf16" else None
    fo = ssd_ref.stack_fwd(x0, layers, segment=seg, store=store)
    bo = ssd_ref.stack_bwd(fo["xs"], layers, dout, store=store)
    tol = stack_tol(dtype, cfg.nlayers) if dtype == "bf16" else TOL[dtype]
    check("out", host(f["out"]), fo["out"], tol)
    check("final_states", host(f["final_states"]), np.stack(fo["final_states"]), tol)
    check("s_ckpt", host(f["s_ckpt"]), np.stack(fo["boundary_states"]), tol)
    check("dx0", host(b["dx0"]), bo["dx0"], tol)
    for k in ("ddt", "dA", "dB", "dC", "dD"):
        check(k, host(b[k]), np.stack([g[k] for g in bo["grads"]]), tol)


def test_stack_grid_choice_does_not_change_results():
    cfg = synth.SSDConfig("stack", "f32", 2, 256, 2, 16, 16, 1, 32, 64, nlayers=4, index=61)
    x0, dout, layers = stack_inputs(cfg)
    f1, b1 = run_stack(cfg, x0, dout, layers, 4, 256)
    f2, b2 = run_stack(cfg, x0, dout, layers, 2, 64)
    f3, b3 = run_stack(cfg, x0, dout, layers, 1, 32)
    assert torch.equal(f1["out"], f2["out"]) and torch.equal(f1["out"], f3["out"])
    for k in ("dx0", "ddt", "dB", "dC"):
        assert torch.equal(b1[k], b2[k]) and torch.equal(b1[k], b3[k]), k
    for k in ("dA", "dD"):
        assert torch.allclose(b1[k], b2[k], rtol=1e-5, atol=1e-6) and torch.allclose(b1[k], b3[k], rtol=1e-5, atol=1e-6)
