"""TEST INFRASTRUCTURE ONLY -- fp64 numpy definition of the block's causal depthwise convolution
(kernel 4) + bias + SiLU and of its reverse mode, with the three-token state that a sequence
checkpoint carries next to the SSM state (App. C, Tab. 7).

Only tests, the smoke check and benchmark baselines may import this.

    upad = [state_in (3 rows, zeros if absent) ; u]
    pre[t, c] = bias[c] + sum_{k=0..3} w[c, k] upad[t + k, c]         (t = 0 .. L-1)
    out = pre * sigmoid(pre);   state_out = last three rows of upad
"""
from __future__ import annotations

import numpy as np


def _pad(u, state_in):
    Bt, L, C = u.shape
    s = np.zeros((Bt, 3, C)) if state_in is None else np.asarray(state_in, dtype=np.float64)
    return np.concatenate([s, np.asarray(u, dtype=np.float64)], axis=1)


def conv1d_silu_fwd(u, w, bias=None, state_in=None):
    """Returns dict(out [Bt,L,C], state_out [Bt,3,C], pre)."""
    w = np.asarray(w, dtype=np.float64)
    Bt, L, C = u.shape
    up = _pad(u, state_in)
    pre = np.zeros((Bt, L, C)) + (0.0 if bias is None else np.asarray(bias, dtype=np.float64))
    for k in range(4):
        pre = pre + w[:, k] * up[:, k:k + L]
    sig = 1.0 / (1.0 + np.exp(-pre))
    return {"out": pre * sig, "state_out": up[:, L:L + 3].copy(), "pre": pre}


def conv1d_silu_bwd(u, w, bias, state_in, dout, dstate_out=None):
    """Gradients of <dout, out> + <dstate_out, state_out>: dict(du, dw [C,4], dbias [C], dstate_in [Bt,3,C])."""
    w = np.asarray(w, dtype=np.float64)
    Bt, L, C = u.shape
    up = _pad(u, state_in)
    pre = conv1d_silu_fwd(u, w, bias, state_in)["pre"]
    sig = 1.0 / (1.0 + np.exp(-pre))
    g = np.asarray(dout, dtype=np.float64) * sig * (1.0 + pre * (1.0 - sig))
    dup = np.zeros_like(up)
    dw = np.zeros((C, 4))
    for k in range(4):
        dup[:, k:k + L] += w[:, k] * g
        dw[:, k] = np.sum(g * up[:, k:k + L], axis=(0, 1))
    if dstate_out is not None:
        dup[:, L:L + 3] += np.asarray(dstate_out, dtype=np.float64)
    return {"du": dup[:, 3:], "dw": dw, "dbias": g.sum(axis=(0, 1)), "dstate_in": dup[:, :3]}
