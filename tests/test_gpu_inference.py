"""GPU parity of the forward-only uses of the path against the fp64 oracle of the plain recurrence
(Sec. 3.1, Eq. 1): prefill without checkpoints (memory independent of the sequence length) and the
token-by-token recurrent step that continues from the prefill's final state."""
import numpy as np
import pytest
import torch

import paper_2411_19460_amd as pk
from oracle import ssd_ref
from paper_2411_19460_amd import synth
from parity_util import TOL, check, dev_inputs, host

pytestmark = pytest.mark.gpu


def _inputs(seed, dtype, Bt, L, H, P, G, N):
    cfg = synth.SSDConfig("t", dtype, Bt, L, H, P, N, G, 1, L, index=70 + seed)
    return synth.make_layer_inputs(cfg, with_states=True)


def _slice_tokens(d, lo, hi):
    return {k: (v[:, lo:hi].contiguous() if k in ("x", "dt", "B", "C") else v) for k, v in d.items()}


@pytest.mark.parametrize("case", [
    # dtype, Bt, L,   H, P,  G, N,   Q,   segment, flags
    ("f32", 2, 256, 4, 16, 2, 16, 64, 64, 0),
    ("bf16", 2, 1024, 4, 64, 2, 128, 256, 256, 0),
    ("bf16", 1, 1024, 2, 64, 1, 128, 128, 256, pk.SSD_FLAG_GENERIC_KERNELS),
])
def test_prefill_without_checkpoints_equals_checkpointed_forward(case):
    dtype, Bt, L, H, P, G, N, Q, seg, flags = case
    dv = dev_inputs(_inputs(1, dtype, Bt, L, H, P, G, N), dtype)
    args = (dv["x"], dv["dt"], dv["A"], dv["B"], dv["C"], dv["D"], Q, seg, dv["init_state"], flags)
    y1, fin1, bnd1 = pk.ssd_fwd(*args)
    y2, fin2, bnd2 = pk.ssd_fwd(*args, want_boundary=False)
    torch.cuda.synchronize()
    assert bnd1 is not None and bnd2 is None
    assert torch.equal(y1, y2) and torch.equal(fin1, fin2)


def test_prefill_workspace_does_not_grow_with_the_sequence():
    a = pk.ssd_shape_t(pk.SSD_BF16, 80, 64, 1, 128, 256, 1, 1 << 16, 4096, 0, 0, 0)
    b = pk.ssd_shape_t(pk.SSD_BF16, 80, 64, 1, 128, 256, 1, 1 << 21, 4096, 0, 0, 0)
    assert pk.ssd_workspace_bytes(a, False) == pk.ssd_workspace_bytes(b, False)


@pytest.mark.parametrize("case", [
    # dtype, Bt, L,  T,  H, P,  G, N,   Q,  segment
    ("f32", 2, 128, 7, 4, 16, 2, 16, 64, 64),
    ("f32", 1, 96, 1, 3, 24, 1, 40, 48, 96),
    ("bf16", 2, 512, 5, 4, 64, 2, 128, 256, 256),
])
def test_decode_continues_the_prefill(case):
    dtype, Bt, L, T, H, P, G, N, Q, seg = case
    d = _inputs(2, dtype, Bt, L + T, H, P, G, N)
    dv = dev_inputs(d, dtype)
    pre, post = _slice_tokens(dv, 0, L), _slice_tokens(dv, L, L + T)
    y0, state, _ = pk.ssd_fwd(pre["x"], pre["dt"], pre["A"], pre["B"], pre["C"], pre["D"], Q, seg, dv["init_state"],
                              want_boundary=False)
    y1 = pk.ssd_decode(post["x"], post["dt"], post["A"], post["B"], post["C"], post["D"], state)
    torch.cuda.synchronize()
    f = ssd_ref.ssd_fwd(d["x"], d["dt"], d["A"], d["B"], d["C"], d["D"], d["init_state"])
    tol = TOL[dtype]
    check("y (prefill)", host(y0), f["y"][:, :L], tol)
    check("y (decode)", host(y1), f["y"][:, L:], tol)
    check("state", host(state), f["final_state"], tol)


def test_decode_alone_equals_the_recurrence_and_handles_flags():
    d = _inputs(3, "f32", 2, 40, 3, 8, 3, 12)
    dv = dev_inputs(d, "f32")
    state = dv["init_state"].clone()
    y = pk.ssd_decode(dv["x"], dv["dt"], dv["A"], dv["B"], dv["C"], dv["D"], state)
    state_r = dv["init_state"].clone()
    yr = pk.ssd_decode(dv["x"], dv["dt"], dv["A"], dv["B"], dv["C"], dv["D"], state_r, flags=pk.SSD_FLAG_RESIDUAL)
    # token by token gives what one call gives
    state_1 = dv["init_state"].clone()
    ys = [pk.ssd_decode(dv["x"][:, t:t + 1].contiguous(), dv["dt"][:, t:t + 1].contiguous(), dv["A"],
                        dv["B"][:, t:t + 1].contiguous(), dv["C"][:, t:t + 1].contiguous(), dv["D"], state_1)
          for t in range(40)]
    torch.cuda.synchronize()
    f = ssd_ref.ssd_fwd(d["x"], d["dt"], d["A"], d["B"], d["C"], d["D"], d["init_state"])
    check("y", host(y), f["y"], TOL["f32"])
    check("state", host(state), f["final_state"], TOL["f32"])
    check("y residual", host(yr), f["y"] + d["x"], TOL["f32"])
    assert torch.equal(torch.cat(ys, dim=1), y) and torch.equal(state_1, state)
    # zero tokens: nothing is touched
    empty = {k: dv[k][:, :0].contiguous() for k in ("x", "dt", "B", "C")}
    before = state.clone()
    pk.ssd_decode(empty["x"], empty["dt"], dv["A"], empty["B"], empty["C"], dv["D"], state)
    torch.cuda.synchronize()
    assert torch.equal(before, state)


def test_layer_shape_2p7b_prefill_then_decode_sampled_heads():
    # the 2.7B layer shape: 16384-token prefill in 4096-token segments without checkpoints, then 3 decoded tokens
    L, T = 16384, 3
    cfg = synth.CONFIGS[2]
    dev = torch.device("cuda:0")
    full = synth.make_layer_inputs_device(synth.CONFIGS[2].scaled(seqlen=L + 4096, name="c2_prefill"), dev, with_dy=False)
    pre = {k: (v[:, :L].contiguous() if k in ("x", "dt", "B", "C") else v) for k, v in full.items()}
    post = {k: (v[:, L:L + T].contiguous() if k in ("x", "dt", "B", "C") else v) for k, v in full.items()}
    y0, state, _ = pk.ssd_fwd(pre["x"], pre["dt"], pre["A"], pre["B"], pre["C"], pre["D"], cfg.chunk, cfg.segment,
                              want_boundary=False)
    y1 = pk.ssd_decode(post["x"], post["dt"], post["A"], post["B"], post["C"], post["D"], state)
    torch.cuda.synchronize()
    heads = [0, 41, 79]
    hs = torch.tensor(heads, device=dev)
    sub = {k: host(full[k][:, :L + T].index_select(2, hs)) for k in ("x", "dt")}
    sub.update({k: host(full[k].index_select(0, hs)) for k in ("A", "D")})
    sub.update({k: host(full[k][:, :L + T]) for k in ("B", "C")})
    f = ssd_ref.ssd_fwd(sub["x"], sub["dt"], sub["A"], sub["B"], sub["C"], sub["D"])
    tol = TOL["bf16"]
    check("y (prefill)", host(y0.index_select(2, hs)), f["y"][:, :L], tol)
    check("y (decode)", host(y1.index_select(2, hs)), f["y"][:, L:], tol)
    check("state", host(state.index_select(1, hs)), f["final_state"], tol)
