"""TEST INFRASTRUCTURE ONLY -- fp64 definition of the block's two projections (dense layers without bias:
the input projection in front of the convolution and the output projection behind the gated
normalisation of the Mamba-2 block that is the backbone of Sec. 3.1; App. C, Tab. 7 sizes the
grid-cell activations by the input projection's width) and of their reverse mode.

Only tests, the smoke check and benchmark baselines may import this.

    out[t, o] = sum_i x[t, i] w[o, i]
"""
from __future__ import annotations

import numpy as np


def linear_fwd(x, w):
    """x [T, I], w [O, I] -> out [T, O] (fp64)."""
    return np.asarray(x, dtype=np.float64) @ np.asarray(w, dtype=np.float64).T


def linear_bwd(x, w, dout):
    """Gradients of <dout, out>: dict(dx [T, I], dw [O, I])."""
    x, w, dout = (np.asarray(a, dtype=np.float64) for a in (x, w, dout))
    return {"dx": dout @ w, "dw": dout.T @ x}
