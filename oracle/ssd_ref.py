"""TEST INFRASTRUCTURE ONLY -- Python face of the fp64 CPU oracle.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this.
It loads `libssd_oracle.so` (plain C, built from `ssd_oracle.c` by `oracle/build.py`)
through ctypes and adds the residual stack of SSD layers on top of it.

Single layer (paper Sec. 3.1, Eq. 1 in the Mamba-2 form):
    h_t = exp(dt_t A) h_{t-1} + dt_t x_t (x) B_t,   y_t = C_t h_t + D x_t
Stack (the layer axis of the paper's Sec. 3.2 grid): x_{j+1} = x_j + SSD_j(x_j),
every layer followed by its residual add, output = x_nlayers.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None
_dp = ctypes.POINTER(ctypes.c_double)
_ip = ctypes.POINTER(ctypes.c_int)


def _lib():
    global _LIB
    if _LIB is None:
        path = os.path.join(_HERE, "libssd_oracle.so")
        if not os.path.exists(path):
            from . import build as _build
            _build.build()
        lib = ctypes.CDLL(path)
        lib.ssd_oracle_fwd.restype = ctypes.c_int
        lib.ssd_oracle_fwd.argtypes = [ctypes.c_long, ctypes.c_long] + [ctypes.c_int] * 4 + [_dp] * 7 + [
            _ip, _dp, _dp, ctypes.c_long, _dp]
        lib.ssd_oracle_bwd.restype = ctypes.c_int
        lib.ssd_oracle_bwd.argtypes = [ctypes.c_long, ctypes.c_long] + [ctypes.c_int] * 4 + [_dp] * 7 + [
            _ip, _dp, _dp] + [_dp] * 7 + [ctypes.c_long]
        _bp = ctypes.POINTER(ctypes.c_ubyte)
        lib.ssd_oracle_fwd_packed.restype = ctypes.c_int
        lib.ssd_oracle_fwd_packed.argtypes = [ctypes.c_long, ctypes.c_long] + [ctypes.c_int] * 4 + [_dp] * 7 + [
            _ip, _bp, _dp, _dp, ctypes.c_long, _dp]
        lib.ssd_oracle_bwd_packed.restype = ctypes.c_int
        lib.ssd_oracle_bwd_packed.argtypes = [ctypes.c_long, ctypes.c_long] + [ctypes.c_int] * 4 + [_dp] * 7 + [
            _ip, _bp, _dp, _dp] + [_dp] * 7 + [ctypes.c_long]
        _LIB = lib
    return _LIB


def _f64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def _p(a):
    return None if a is None else a.ctypes.data_as(_dp)


def _dims(x, Bm):
    Bt, L, H, P = x.shape
    G, N = Bm.shape[2], Bm.shape[3]
    return Bt, L, H, P, G, N


def _reset_ptr(reset, Bt, L):
    if reset is None:
        return None, None
    r = np.ascontiguousarray(reset, dtype=np.uint8)
    assert r.shape == (Bt, L)
    return r, r.ctypes.data_as(ctypes.POINTER(ctypes.c_ubyte))


def ssd_fwd(x, dt, A, B, C, D, init_state=None, segment=None, head_group=None, reset=None):
    """Returns dict(y, final_state, boundary_states) in fp64.

    boundary_states[b, k] = state entering segment k (k = 0 is the initial state);
    it is None when `segment` is None.  reset [Bt, L] (0/1), optional: packed sequences -- a token with
    reset = 1 starts a new sequence and sees no state from the tokens before it."""
    x, dt, A, B, C, D, init_state = map(_f64, (x, dt, A, B, C, D, init_state))
    Bt, L, H, P, G, N = _dims(x, B)
    hg = None if head_group is None else np.ascontiguousarray(head_group, dtype=np.int32)
    y = np.empty_like(x)
    fin = np.empty((Bt, H, P, N))
    bnd = None
    if segment is not None:
        assert L % segment == 0
        bnd = np.empty((Bt, L // segment, H, P, N))
    keep, rp = _reset_ptr(reset, Bt, L)
    rc = _lib().ssd_oracle_fwd_packed(Bt, L, H, P, G, N, _p(x), _p(dt), _p(A), _p(B), _p(C), _p(D), _p(init_state),
                                      None if hg is None else hg.ctypes.data_as(_ip), rp, _p(y), _p(fin),
                                      0 if segment is None else segment, _p(bnd))
    if rc != 0:
        raise RuntimeError(f"ssd_oracle_fwd failed: {rc}")
    return {"y": y, "final_state": fin, "boundary_states": bnd}


def ssd_bwd(x, dt, A, B, C, D, dy, init_state=None, dfinal_state=None, head_group=None, ckpt_every=256, reset=None):
    """Reverse-mode gradients of <dy, y> + <dfinal_state, final_state>, fp64."""
    x, dt, A, B, C, D, dy, init_state, dfinal_state = map(
        _f64, (x, dt, A, B, C, D, dy, init_state, dfinal_state))
    Bt, L, H, P, G, N = _dims(x, B)
    hg = None if head_group is None else np.ascontiguousarray(head_group, dtype=np.int32)
    dx = np.empty_like(x)
    ddt = np.empty_like(dt)
    dA = np.empty(H)
    dD = np.empty(H)
    dB = np.empty_like(B)
    dC = np.empty_like(C)
    dinit = np.empty((Bt, H, P, N))
    keep, rp = _reset_ptr(reset, Bt, L)
    rc = _lib().ssd_oracle_bwd_packed(Bt, L, H, P, G, N, _p(x), _p(dt), _p(A), _p(B), _p(C), _p(D), _p(init_state),
                                      None if hg is None else hg.ctypes.data_as(_ip), rp, _p(dy), _p(dfinal_state),
                                      _p(dx), _p(ddt), _p(dA), _p(dB), _p(dC), _p(dD), _p(dinit), ckpt_every)
    if rc != 0:
        raise RuntimeError(f"ssd_oracle_bwd failed: {rc}")
    return {"dx": dx, "ddt": ddt, "dA": dA, "dB": dB, "dC": dC, "dD": dD, "dinit_state": dinit}


def stack_fwd(x0, layers, init_states=None, segment=None, head_group=None, store=None, progress=None):
    """Residual stack: x_{j+1} = x_j + SSD_j(x_j).  `layers` is a list of dicts with
    dt, A, B, C, D.  `store`, if given, is the rounding of the storage dtype (e.g. round to
    bf16): the stack keeps its activations in that dtype, so every x_{j+1} is rounded once
    when it is stored; with store=None everything stays in fp64 between layers.
    `progress`, if given, is called with a short text after every layer (long runs report their steps).
    Returns dict(out, xs=[x_0..x_{n-1}], final_states, boundary_states)."""
    x = _f64(x0)
    xs, fins, bnds = [], [], []
    for j, lay in enumerate(layers):
        xs.append(x)
        r = ssd_fwd(x, lay["dt"], lay["A"], lay["B"], lay["C"], lay["D"],
                    None if init_states is None else init_states[j], segment, head_group)
        x = x + r["y"]
        if store is not None:
            x = _f64(store(x))
        fins.append(r["final_state"])
        bnds.append(r["boundary_states"])
        if progress is not None:
            progress(f"stack oracle: forward layer {j} done")
    return {"out": x, "xs": xs, "final_states": fins, "boundary_states": bnds}


def stack_bwd(xs, layers, dout, init_states=None, dfinal_states=None, head_group=None, store=None, progress=None):
    """Backward of stack_fwd given the layer inputs xs[j]: dx_j = dx_{j+1} + VJP_j(dx_{j+1}),
    each dx_j rounded once by `store` (the storage dtype of the activation gradients) if given.
    Returns dict(dx0, grads=[per-layer dict of ddt, dA, dB, dC, dD, dinit_state], dys=[gradient entering layer j])."""
    g = _f64(dout)
    grads = [None] * len(layers)
    dys = [None] * len(layers)
    for j in range(len(layers) - 1, -1, -1):
        lay = layers[j]
        dys[j] = g
        r = ssd_bwd(xs[j], lay["dt"], lay["A"], lay["B"], lay["C"], lay["D"], g,
                    None if init_states is None else init_states[j],
                    None if dfinal_states is None else dfinal_states[j], head_group)
        g = g + r.pop("dx")
        if store is not None:
            g = _f64(store(g))
        grads[j] = r
        if progress is not None:
            progress(f"stack oracle: backward layer {j} done")
    return {"dx0": g, "grads": grads, "dys": dys}
