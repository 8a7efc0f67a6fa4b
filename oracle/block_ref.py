"""TEST INFRASTRUCTURE ONLY -- fp64 definition of one Mamba-2 block (the backbone layer of Sec. 3.1 whose
per-token activations and per-checkpoint states App. C, Tab. 7 counts) as the composition of the pieces
defined next to this file, and of its reverse mode:

    zxbcdt = u W_in^T                      [L, 2 d_inner + 2 G N + H]  = (z | xBC | dt_raw)
    xBC    = silu(causal depthwise conv4(xBC) + bias)            (three-token state)
    dt     = softplus(dt_raw + dt_bias)
    y      = SSD(x, dt, A, B, C, D)   with (x | B | C) = xBC      (SSM state)
    out    = RMSNorm_G(y * silu(z)) * norm_w  W_out^T
With the optional parameter pre_norm_w the projection reads RMSNorm(u) * pre_norm_w instead of u: together
with the residual add of the stack below that is the pre-norm layer of the language model.

Only tests, the smoke check and benchmark baselines may import this.

`store`, if given, is the rounding of the storage dtype: every intermediate tensor that the device path
keeps in memory between two steps (the normalised input, zxbcdt, xBC, dt, y, the normalised y, out, and in the backward sweep
the gradients of the same tensors) is rounded once where it is stored; with store=None everything stays fp64.
One sequence (batch 1).
"""
from __future__ import annotations

import numpy as np

from . import conv_ref, linear_ref, norm_ref, ssd_ref


def _st(store, a):
    return a if store is None else np.asarray(store(a), dtype=np.float64)


def dims(p, H, P, G, N):
    d_inner = H * P
    conv_dim = d_inner + 2 * G * N
    return d_inner, conv_dim, 2 * d_inner + 2 * G * N + H


def block_fwd(u, p, H, P, G, N, eps=1e-5, conv_state=None, ssm_state=None, store=None):
    """u [L, d_model]; p: W_in, conv_w, conv_b, dt_bias, A, D, norm_w, W_out and, optionally, pre_norm_w (then the
    input projection reads RMSNorm(u) * pre_norm_w: the pre-norm of a language-model layer).  Returns dict with out and
    every intermediate (for the backward pass), plus the states leaving the sequence."""
    L = u.shape[0]
    d_inner, conv_dim, d_in_proj = dims(p, H, P, G, N)
    un = u if p.get("pre_norm_w") is None else _st(store, norm_ref.gated_rmsnorm_fwd(u, None, p["pre_norm_w"], eps, 1))
    zx = _st(store, linear_ref.linear_fwd(un, p["W_in"]))
    z, pre, dt_raw = zx[:, :d_inner], zx[:, d_inner:d_inner + conv_dim], zx[:, d_inner + conv_dim:]
    c = conv_ref.conv1d_silu_fwd(pre[None], p["conv_w"], p["conv_b"], None if conv_state is None else conv_state[None])
    xBC = _st(store, c["out"][0])
    v = dt_raw + np.asarray(p["dt_bias"], dtype=np.float64)
    dt = _st(store, np.logaddexp(0.0, v))
    x = xBC[:, :d_inner].reshape(1, L, H, P)
    Bm = xBC[:, d_inner:d_inner + G * N].reshape(1, L, G, N)
    Cm = xBC[:, d_inner + G * N:].reshape(1, L, G, N)
    r = ssd_ref.ssd_fwd(x, dt[None], p["A"], Bm, Cm, p["D"], None if ssm_state is None else ssm_state[None])
    y = _st(store, r["y"][0].reshape(L, d_inner))
    yn = _st(store, norm_ref.gated_rmsnorm_fwd(y, z, p["norm_w"], eps, G))
    out = _st(store, linear_ref.linear_fwd(yn, p["W_out"]))
    return {"out": out, "un": un, "zxbcdt": zx, "xBC": xBC, "dt": dt, "y": y, "yn": yn,
            "conv_state": c["state_out"][0], "ssm_state": r["final_state"][0]}


def block_bwd(u, p, H, P, G, N, dout, eps=1e-5, conv_state=None, ssm_state=None, dconv_state=None, dssm_state=None,
              store=None):
    """Gradients of <dout, out> + <dconv_state, conv_state_out> + <dssm_state, ssm_state_out>:
    dict(du, dW_in, dconv_w, dconv_b, ddt_bias, dA, dD, dnorm_w, dW_out, dconv_state_in, dssm_state_in)."""
    L = u.shape[0]
    d_inner, conv_dim, d_in_proj = dims(p, H, P, G, N)
    f = block_fwd(u, p, H, P, G, N, eps, conv_state, ssm_state, store)
    zx = f["zxbcdt"]
    z, pre, dt_raw = zx[:, :d_inner], zx[:, d_inner:d_inner + conv_dim], zx[:, d_inner + conv_dim:]
    go = linear_ref.linear_bwd(f["yn"], p["W_out"], dout)
    dyn = _st(store, go["dx"])
    gn = norm_ref.gated_rmsnorm_bwd(f["y"], z, p["norm_w"], dyn, eps, G)
    dy, dz = _st(store, gn["dy"]), _st(store, gn["dz"])
    x = f["xBC"][:, :d_inner].reshape(1, L, H, P)
    Bm = f["xBC"][:, d_inner:d_inner + G * N].reshape(1, L, G, N)
    Cm = f["xBC"][:, d_inner + G * N:].reshape(1, L, G, N)
    gs = ssd_ref.ssd_bwd(x, f["dt"][None], p["A"], Bm, Cm, p["D"], dy.reshape(1, L, H, P),
                         None if ssm_state is None else ssm_state[None], None if dssm_state is None else dssm_state[None])
    dxBC = _st(store, np.concatenate([gs["dx"][0].reshape(L, d_inner), gs["dB"][0].reshape(L, G * N),
                                      gs["dC"][0].reshape(L, G * N)], axis=1))
    ddt = _st(store, gs["ddt"][0])
    v = dt_raw + np.asarray(p["dt_bias"], dtype=np.float64)
    draw = ddt / (1.0 + np.exp(-v))                      # d softplus = sigmoid
    gc = conv_ref.conv1d_silu_bwd(pre[None], p["conv_w"], p["conv_b"], None if conv_state is None else conv_state[None],
                                  dxBC[None], None if dconv_state is None else dconv_state[None])
    dzx = _st(store, np.concatenate([dz, gc["du"][0], draw], axis=1))
    gi = linear_ref.linear_bwd(f["un"], p["W_in"], dzx)
    du, extra = _st(store, gi["dx"]), {}
    if p.get("pre_norm_w") is not None:   # back through the normalisation in front of the projection
        gp = norm_ref.gated_rmsnorm_bwd(u, None, p["pre_norm_w"], du, eps, 1)
        du, extra = _st(store, gp["dy"]), {"dpre_norm_w": gp["dw"]}
    return {**extra, "du": du, "dW_in": gi["dw"], "dconv_w": gc["dw"], "dconv_b": gc["dbias"],
            "ddt_bias": draw.sum(axis=0), "dA": gs["dA"], "dD": gs["dD"], "dnorm_w": gn["dw"], "dW_out": go["dw"],
            "dconv_state_in": gc["dstate_in"][0], "dssm_state_in": gs["dinit_state"][0]}


def stack_fwd(x0, layers, H, P, G, N, eps=1e-5, store=None, conv_states=None, ssm_states=None):
    """Residual stack of blocks: x_{j+1} = x_j + Block_j(x_j); `layers` is a list of parameter dicts, the
    states entering the sequence are given per layer (None = zeros).  Every x_{j+1} is rounded once by
    `store` where it is stored.  Returns dict(out, xs, conv_states, ssm_states): the last two are the states
    of every layer behind the last token (what a later call continues from)."""
    x = np.asarray(x0, dtype=np.float64)
    xs, cs, ss = [], [], []
    for j, p in enumerate(layers):
        xs.append(x)
        f = block_fwd(x, p, H, P, G, N, eps, None if conv_states is None else conv_states[j],
                      None if ssm_states is None else ssm_states[j], store=store)
        cs.append(f["conv_state"])
        ss.append(f["ssm_state"])
        x = _st(store, x + f["out"])
    return {"out": x, "xs": xs, "conv_states": cs, "ssm_states": ss}


def stack_bwd(xs, layers, H, P, G, N, dout, eps=1e-5, store=None):
    """Backward of stack_fwd given the layer inputs: dx_j = dx_{j+1} + Block_j^T(dx_{j+1}), each rounded once
    by `store`.  Returns dict(dx0, grads=[per-layer dict])."""
    g = np.asarray(dout, dtype=np.float64)
    grads = [None] * len(layers)
    for j in range(len(layers) - 1, -1, -1):
        r = block_bwd(xs[j], layers[j], H, P, G, N, g, eps, store=store)
        g = _st(store, g + r.pop("du"))
        grads[j] = r
    return {"dx0": g, "grads": grads}
