"""GPU parity of the block's causal depthwise convolution + SiLU (forward, backward, state hand-over
between segments) against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2411_19460_amd as pk
from oracle import conv_ref
from paper_2411_19460_amd import synth
from parity_util import TOL, check, host

pytestmark = pytest.mark.gpu


def draw(seed, dtype, Bt, L, C):
    r = np.random.default_rng(1000 + seed)
    rnd = synth.round_bf16 if dtype == "bf16" else (lambda a: a.astype(np.float32).astype(np.float64))
    return dict(u=rnd(r.standard_normal((Bt, L, C))), w=r.standard_normal((C, 4)).astype(np.float32).astype(np.float64) * 0.5,
                bias=r.standard_normal(C).astype(np.float32).astype(np.float64), state_in=rnd(r.standard_normal((Bt, 3, C))),
                dout=rnd(r.standard_normal((Bt, L, C))),
                dstate_out=r.standard_normal((Bt, 3, C)).astype(np.float32).astype(np.float64))


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16) if dtype == "bf16" else t


@pytest.mark.parametrize("case", [
    # dtype, Bt, L,   C
    ("bf16", 2, 1000, 5376),     # the 2.7B block's convolution width (d_inner + 2 G N), ragged length
    ("bf16", 1, 300, 37),        # channel count not a multiple of the vector width
    ("f32", 2, 515, 64),
    ("f32", 1, 70, 5),
    ("bf16", 2, 2, 16),          # shorter than the kernel: part of the state passes through
    ("f32", 1, 0, 8),            # empty segment: the state passes through untouched
])
def test_conv_forward_backward(case):
    dtype, Bt, L, C = case
    d = draw(1, dtype, Bt, L, C)
    u, st, dout = dev(d["u"], dtype), dev(d["state_in"], dtype), dev(d["dout"], dtype)
    w, bias, dso = dev(d["w"]), dev(d["bias"]), dev(d["dstate_out"])
    out, so = pk.ssd_conv1d_fwd(u, w, bias, st)
    g = pk.ssd_conv1d_bwd(u, w, bias, st, dout, dso)
    torch.cuda.synchronize()
    f = conv_ref.conv1d_silu_fwd(d["u"], d["w"], d["bias"], d["state_in"])
    go = conv_ref.conv1d_silu_bwd(d["u"], d["w"], d["bias"], d["state_in"], d["dout"], d["dstate_out"])
    tol = TOL[dtype]
    if L:
        check("out", host(out), f["out"], tol)
        check("du", host(g["du"]), go["du"], tol)
    assert np.array_equal(host(so), f["state_out"])          # a copy of stored values: exact
    check("dstate_in", host(g["dstate_in"]), go["dstate_in"], tol)
    check("dw", host(g["dw"]), go["dw"], tol)
    check("dbias", host(g["dbias"]), go["dbias"], tol)


def test_segments_chained_through_the_state_equal_one_call_and_gradients_accumulate():
    dtype, Bt, L, C, s = "bf16", 2, 1536, 256, 512
    d = draw(2, dtype, Bt, L, C)
    u, st, dout = dev(d["u"], dtype), dev(d["state_in"], dtype), dev(d["dout"], dtype)
    w, bias, dso = dev(d["w"]), dev(d["bias"]), dev(d["dstate_out"])
    out, so = pk.ssd_conv1d_fwd(u, w, bias, st)
    g = pk.ssd_conv1d_bwd(u, w, bias, st, dout, dso)
    # forward: segment by segment, keeping the state entering each (the checkpoint)
    states, outs, cur = [], [], st
    for k in range(L // s):
        states.append(cur)
        o, cur = pk.ssd_conv1d_fwd(u[:, k * s:(k + 1) * s].contiguous(), w, bias, cur)
        outs.append(o)
    assert torch.equal(torch.cat(outs, dim=1), out) and torch.equal(cur, so)
    # backward: right to left, restarting every segment from its checkpoint, parameter gradients accumulated
    dw = torch.zeros_like(g["dw"])
    db = torch.zeros_like(g["dbias"])
    carry, dus = dso, []
    for k in reversed(range(L // s)):
        gk = pk.ssd_conv1d_bwd(u[:, k * s:(k + 1) * s].contiguous(), w, bias, states[k], dout[:, k * s:(k + 1) * s].contiguous(),
                               carry, flags=pk.SSD_FLAG_ACCUM_PARAM, dw=dw, dbias=db)
        carry = gk["dstate_in"]
        dus.insert(0, gk["du"])
    torch.cuda.synchronize()
    assert torch.equal(torch.cat(dus, dim=1), g["du"])
    check("dstate_in", host(carry), host(g["dstate_in"]), 1e-6)
    check("dw", host(dw), host(g["dw"]), 1e-5)
    check("dbias", host(db), host(g["dbias"]), 1e-5)
