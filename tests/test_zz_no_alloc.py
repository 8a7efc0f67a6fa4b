"""ssd_fwd_static (the forward pass for callers that cannot allocate: scratch in the library's own device
array) against ssd_fwd with a caller's workspace, through the C ABI: two calls in a row, the second on a
smaller input, so that the array still holds the first call's contents when the second one runs."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2411_19460_amd as pk
from paper_2411_19460_amd import binding, synth

pytestmark = pytest.mark.gpu


def _inputs(cfg):
    d = synth.make_layer_inputs(cfg)
    td = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    return {k: torch.from_numpy(v).cuda().to(torch.float32 if k in ("A", "D") else td) for k, v in d.items()}


def _both(cfg):
    dv = _inputs(cfg)
    args = (dv["x"], dv["dt"], dv["A"], dv["B"], dv["C"], dv["D"], cfg.chunk, cfg.segment)
    y0, fin0, bnd0 = pk.ssd_fwd(*args)
    out = {"y": torch.full_like(y0, float("nan")), "final_state": torch.full_like(fin0, float("nan")),
           "boundary_states": torch.full_like(bnd0, float("nan"))}
    before = torch.cuda.memory_allocated()
    y1, fin1, bnd1 = pk.ssd_fwd_static(*args, out=out)
    assert torch.cuda.memory_allocated() == before      # the binding allocated nothing either
    torch.cuda.synchronize()
    for name, a, b in (("y", y0, y1), ("final_state", fin0, fin1), ("boundary_states", bnd0, bnd1)):
        a, b = a.float().cpu().numpy(), b.float().cpu().numpy()
        assert np.all(np.isfinite(b)), name
        scale = max(float(np.max(np.abs(a))), 1e-30)
        err = float(np.max(np.abs(a - b))) / scale
        tol = 2e-2 if cfg.dtype == "bf16" else 1e-3
        assert err <= tol, f"{cfg.name}.{name}: {err:.3e}"
        # the two entry points run the same kernels on the same values: the results are in fact identical
        assert np.array_equal(a, b), f"{cfg.name}.{name}: not bit-equal (err {err:.3e})"


def test_static_scratch_forward_matches_workspace_forward_twice():
    pk.ssd_init()
    big = synth.SSDConfig("static_big", "bf16", 1, 2560, 8, 64, 128, 1, 256, 1024, index=21)    # 3 segments, last one short
    small = synth.SSDConfig("static_small", "bf16", 1, 700, 3, 64, 128, 1, 128, 256, index=22)  # ragged tail chunk
    _both(big)
    _both(small)
    _both(synth.CONFIGS[0])                                                                     # fp32, shape-generic kernels


def test_static_scratch_rejects_what_does_not_fit():
    x = torch.zeros((1, 65536, 80, 64), dtype=torch.bfloat16, device="cuda")
    Bm = torch.zeros((1, 65536, 1, 128), dtype=torch.bfloat16, device="cuda")
    shape = binding.make_shape(x, Bm, 256, 65536)        # one 65536-token segment: far beyond the array
    need = pk.ssd_fwd_static_bytes(shape)
    assert need > 40 << 20
    dt = torch.zeros((1, 65536, 80), dtype=torch.bfloat16, device="cuda")
    A = torch.zeros(80, device="cuda")
    with pytest.raises(pk.SSDError) as e:
        pk.ssd_fwd_static(x, dt, A, Bm, Bm, A, 256, 65536, out={"y": x})
    assert e.value.status == -5          # SSD_ERR_WORKSPACE, before anything was launched
    shape_ok = binding.make_shape(x, Bm, 256, 4096)      # the benchmark's segment length fits
    assert 0 < pk.ssd_fwd_static_bytes(shape_ok) <= 40 << 20
