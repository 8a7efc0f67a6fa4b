"""TEST INFRASTRUCTURE ONLY -- fp64 numpy definition of the block's gated RMS normalisation (the step
between the SSD output and the output projection of the Mamba-2 block that is the backbone of
Sec. 3.1; its two inputs, the gate z of the input projection and the SSD output y, are the
d_in_proj + d_inner activations per token that C_grid of App. C, Tab. 7 counts) and of its reverse mode.

Only tests, the smoke check and benchmark baselines may import this.

    g = y * z * sigmoid(z)                                   (gate first, then normalise)
    out[t, c] = g[t, c] / sqrt(mean_{c' in group(c)} g[t, c']^2 + eps) * w[c]
The channels are cut into `ngroups` contiguous groups of equal size, each normalised on its own.
z=None takes the gate away (g = y): the plain RMS normalisation that stands in front of each block.
"""
from __future__ import annotations

import numpy as np


def _gate(y, z):
    y = np.asarray(y, dtype=np.float64)
    if z is None:
        return y, None, None, y
    z = np.asarray(z, dtype=np.float64)
    sig = 1.0 / (1.0 + np.exp(-z))
    return y, z, sig, y * z * sig


def gated_rmsnorm_fwd(y, z, w, eps=1e-5, ngroups=1):
    """y, z [T, C]; w [C].  Returns out [T, C] (fp64)."""
    y, z, sig, g = _gate(y, z)
    T, C = g.shape
    gg = g.reshape(T, ngroups, C // ngroups)
    rstd = 1.0 / np.sqrt(np.mean(gg * gg, axis=2, keepdims=True) + eps)
    return (gg * rstd).reshape(T, C) * np.asarray(w, dtype=np.float64)


def gated_rmsnorm_bwd(y, z, w, dout, eps=1e-5, ngroups=1):
    """Gradients of <dout, out>: dict(dy [T,C], dz [T,C], dw [C])."""
    y, z, sig, g = _gate(y, z)
    w = np.asarray(w, dtype=np.float64)
    dout = np.asarray(dout, dtype=np.float64)
    T, C = g.shape
    gs = C // ngroups
    gg = g.reshape(T, ngroups, gs)
    rstd = 1.0 / np.sqrt(np.mean(gg * gg, axis=2, keepdims=True) + eps)
    ghat = gg * rstd
    dghat = (dout * w).reshape(T, ngroups, gs)
    # d/dg of ghat = g * (mean g^2 + eps)^(-1/2):  rstd * (dghat - ghat * mean(dghat * ghat))
    dg = (rstd * (dghat - ghat * np.mean(dghat * ghat, axis=2, keepdims=True))).reshape(T, C)
    dw = np.sum(dout * ghat.reshape(T, C), axis=0)
    if z is None:
        return {"dy": dg, "dz": None, "dw": dw}
    return {"dy": dg * z * sig, "dz": dg * y * sig * (1.0 + z * (1.0 - sig)), "dw": dw}
