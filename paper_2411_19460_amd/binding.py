"""Thin ctypes binding over libssd_magc.so: same names as the C ABI, argument marshalling only.

PyTorch supplies device memory (`tensor.data_ptr()`) and the stream; every step of the
computation runs inside the library's HIP kernels.  There is no CPU fallback: if the
library is missing, loading fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libssd_magc.so")

SSD_F32, SSD_BF16 = 0, 1
SSD_FLAG_RESIDUAL, SSD_FLAG_ACCUM_PARAM, SSD_FLAG_GENERIC_KERNELS, SSD_FLAG_BF16_CHECKPOINTS, SSD_FLAG_FP32_CHUNK_STATES = 1, 2, 4, 8, 16

EXPORTS = ("ssd_workspace_bytes", "ssd_workspace_bytes_flags", "ssd_fwd", "ssd_bwd", "ssd_decode",
           "ssd_init", "ssd_fwd_static_bytes", "ssd_fwd_static",
           "ssd_conv1d_workspace_bytes", "ssd_conv1d_fwd", "ssd_conv1d_bwd",
           "ssd_gated_norm_workspace_bytes", "ssd_gated_norm_fwd", "ssd_gated_norm_bwd", "ssd_linear_fwd", "ssd_linear_bwd",
           "magc_block_workspace_bytes", "magc_block_fwd", "magc_block_bwd",
           "magc_blockstack_workspace_bytes", "magc_blockstack_fwd", "magc_blockstack_bwd", "magc_blockstack_infer", "magc_blockstack_decode",
           "magc_stack_workspace_bytes", "magc_stack_fwd",
           "magc_stack_bwd", "magc_plan", "ssd_strerror", "ssd_prof_enable", "ssd_prof_read", "ssd_prof_kernel_name", "ssd_prof_serialize", "ssd_prof_mfma_peak", "ssd_prof_clock_probe")


class ssd_shape_t(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("nheads", ctypes.c_int32), ("headdim", ctypes.c_int32),
                ("ngroups", ctypes.c_int32), ("dstate", ctypes.c_int32), ("chunk", ctypes.c_int32),
                ("batch", ctypes.c_int64), ("seqlen", ctypes.c_int64), ("segment", ctypes.c_int64),
                ("x_batch_stride", ctypes.c_int64), ("dt_batch_stride", ctypes.c_int64),
                ("bc_batch_stride", ctypes.c_int64), ("seq_reset", ctypes.c_void_p)]


class ssd_conv_shape_t(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("channels", ctypes.c_int32), ("batch", ctypes.c_int64),
                ("seqlen", ctypes.c_int64), ("batch_stride", ctypes.c_int64), ("u_row_stride", ctypes.c_int64)]


class ssd_norm_shape_t(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("dim", ctypes.c_int32), ("ngroups", ctypes.c_int32), ("eps", ctypes.c_float),
                ("rows", ctypes.c_int64), ("y_row_stride", ctypes.c_int64), ("z_row_stride", ctypes.c_int64)]


class magc_block_shape_t(ctypes.Structure):
    _fields_ = [("d_model", ctypes.c_int32), ("nheads", ctypes.c_int32), ("headdim", ctypes.c_int32), ("ngroups", ctypes.c_int32),
                ("dstate", ctypes.c_int32), ("chunk", ctypes.c_int32), ("eps", ctypes.c_float), ("seqlen", ctypes.c_int64),
                ("segment", ctypes.c_int64)]


BLOCK_PARAMS = ("W_in", "conv_w", "conv_b", "dt_bias", "A", "D", "norm_w", "W_out", "pre_norm_w")   # the last one is optional


class magc_block_params_t(ctypes.Structure):
    _fields_ = [(k, ctypes.c_void_p) for k in BLOCK_PARAMS]


class magc_block_grads_t(ctypes.Structure):
    _fields_ = [("d" + k, ctypes.c_void_p) for k in BLOCK_PARAMS]


class magc_blockstack_shape_t(ctypes.Structure):
    _fields_ = [("block", magc_block_shape_t), ("nlayers", ctypes.c_int32), ("layer_interval", ctypes.c_int32)]


class magc_model_t(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int64), ("seqlen", ctypes.c_int64), ("c_lckpt", ctypes.c_double),
                ("c_sckpt", ctypes.c_double), ("c_grid", ctypes.c_double), ("c_state", ctypes.c_double),
                ("s_multiple", ctypes.c_int64), ("budget", ctypes.c_double), ("integer_counts", ctypes.c_int32)]


class magc_plan_t(ctypes.Structure):
    _fields_ = [("l", ctypes.c_int64), ("s", ctypes.c_int64), ("m_lckpt", ctypes.c_double),
                ("m_sckpt", ctypes.c_double), ("m_grid", ctypes.c_double), ("m_state", ctypes.c_double),
                ("m_total", ctypes.c_double), ("regime", ctypes.c_int32), ("fits", ctypes.c_int32)]


class SSDError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status})")


_lib = None


def lib():
    """Loads the shared library (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2411_19460_amd.build` "
                               "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, i32, u32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32, ctypes.c_uint32
        shp = ctypes.POINTER(ssd_shape_t)
        L.ssd_workspace_bytes.restype = sz
        L.ssd_workspace_bytes.argtypes = [shp, i32]
        L.ssd_workspace_bytes_flags.restype = sz
        L.ssd_workspace_bytes_flags.argtypes = [shp, i32, u32]
        L.ssd_fwd.restype = ctypes.c_int
        L.ssd_fwd.argtypes = [shp] + [vp] * 10 + [vp, sz, u32, vp]
        L.ssd_bwd.restype = ctypes.c_int
        L.ssd_bwd.argtypes = [shp] + [vp] * 17 + [vp, sz, u32, vp]
        L.ssd_init.restype = ctypes.c_int
        L.ssd_init.argtypes = []
        L.ssd_fwd_static_bytes.restype = sz
        L.ssd_fwd_static_bytes.argtypes = [shp, u32]
        L.ssd_fwd_static.restype = ctypes.c_int
        L.ssd_fwd_static.argtypes = [shp] + [vp] * 10 + [u32, vp]
        cshp = ctypes.POINTER(ssd_conv_shape_t)
        L.ssd_conv1d_workspace_bytes.restype = sz
        L.ssd_conv1d_workspace_bytes.argtypes = [cshp]
        L.ssd_conv1d_fwd.restype = ctypes.c_int
        L.ssd_conv1d_fwd.argtypes = [cshp] + [vp] * 6 + [vp]
        L.ssd_conv1d_bwd.restype = ctypes.c_int
        L.ssd_conv1d_bwd.argtypes = [cshp] + [vp] * 10 + [vp, sz, u32, vp]
        nshp = ctypes.POINTER(ssd_norm_shape_t)
        L.ssd_gated_norm_workspace_bytes.restype = sz
        L.ssd_gated_norm_workspace_bytes.argtypes = [nshp]
        L.ssd_gated_norm_fwd.restype = ctypes.c_int
        L.ssd_gated_norm_fwd.argtypes = [nshp] + [vp] * 4 + [vp]
        L.ssd_gated_norm_bwd.restype = ctypes.c_int
        L.ssd_gated_norm_bwd.argtypes = [nshp] + [vp] * 7 + [vp, sz, u32, vp]
        i64 = ctypes.c_int64
        L.ssd_linear_fwd.restype = ctypes.c_int
        L.ssd_linear_fwd.argtypes = [i64, i32, i32, vp, i64, vp, vp, i64, vp]
        L.ssd_linear_bwd.restype = ctypes.c_int
        L.ssd_linear_bwd.argtypes = [i64, i32, i32, vp, i64, vp, vp, i64, vp, i64, vp, u32, vp]
        bshp, bpar, bgr = (ctypes.POINTER(t) for t in (magc_block_shape_t, magc_block_params_t, magc_block_grads_t))
        L.magc_block_workspace_bytes.restype = sz
        L.magc_block_workspace_bytes.argtypes = [bshp, i32]
        L.magc_block_fwd.restype = ctypes.c_int
        L.magc_block_fwd.argtypes = [bshp, bpar] + [vp] * 8 + [vp, sz, vp]
        L.magc_block_bwd.restype = ctypes.c_int
        L.magc_block_bwd.argtypes = [bshp, bpar] + [vp] * 9 + [bgr, vp, vp, vp, sz, u32, vp]
        sshp = ctypes.POINTER(magc_blockstack_shape_t)
        L.magc_blockstack_workspace_bytes.restype = sz
        L.magc_blockstack_workspace_bytes.argtypes = [sshp, i32]
        L.magc_blockstack_fwd.restype = ctypes.c_int
        L.magc_blockstack_fwd.argtypes = [sshp, bpar] + [vp] * 5 + [vp, sz, vp]
        L.magc_blockstack_infer.restype = ctypes.c_int
        L.magc_blockstack_infer.argtypes = [sshp, bpar] + [vp] * 4 + [i32, vp, sz, vp]
        L.magc_blockstack_decode.restype = ctypes.c_int
        L.magc_blockstack_decode.argtypes = [sshp, bpar, i32] + [vp] * 4 + [vp, sz, vp]
        L.magc_blockstack_bwd.restype = ctypes.c_int
        L.magc_blockstack_bwd.argtypes = [sshp, bpar] + [vp] * 6 + [bgr, vp, sz, u32, vp]
        L.ssd_prof_mfma_peak.restype = ctypes.c_int
        L.ssd_prof_mfma_peak.argtypes = [i32, i32, vp, vp]
        L.ssd_decode.restype = ctypes.c_int
        L.ssd_decode.argtypes = [shp] + [vp] * 8 + [u32, vp]
        L.magc_stack_workspace_bytes.restype = sz
        L.magc_stack_workspace_bytes.argtypes = [shp, i32, i32, i32]
        L.magc_stack_fwd.restype = ctypes.c_int
        L.magc_stack_fwd.argtypes = [shp, i32, i32] + [vp] * 10 + [vp, sz, vp]
        L.magc_stack_bwd.restype = ctypes.c_int
        L.magc_stack_bwd.argtypes = [shp, i32, i32] + [vp] * 15 + [vp, sz, vp]
        L.magc_plan.restype = ctypes.c_int
        L.magc_plan.argtypes = [ctypes.POINTER(magc_model_t), ctypes.POINTER(magc_plan_t)]
        L.ssd_prof_enable.restype = ctypes.c_int
        L.ssd_prof_enable.argtypes = [i32]
        L.ssd_prof_serialize.restype = ctypes.c_int
        L.ssd_prof_serialize.argtypes = [i32]
        L.ssd_prof_read.restype = ctypes.c_int
        L.ssd_prof_read.argtypes = [i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
        L.ssd_prof_kernel_name.restype = ctypes.c_char_p
        L.ssd_prof_kernel_name.argtypes = [i32]
        L.ssd_strerror.restype = ctypes.c_char_p
        L.ssd_strerror.argtypes = [ctypes.c_int]
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().ssd_strerror(int(status)).decode()


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(t) -> Optional[int]:
    import torch
    return torch.cuda.current_stream(t.device).cuda_stream or None


def make_shape(x, Bm, chunk: int, segment: Optional[int] = None, seq_reset=None) -> ssd_shape_t:
    import torch
    Bt, L, H, P = x.shape
    G, N = Bm.shape[2], Bm.shape[3]
    if x.dtype == torch.bfloat16:
        dt = SSD_BF16
    elif x.dtype == torch.float32:
        dt = SSD_F32
    else:
        raise TypeError(f"unsupported dtype {x.dtype}")
    if segment is None:   # one segment: the sequence rounded up to whole chunks
        segment = max(chunk, -(-L // chunk) * chunk)
    if seq_reset is not None:
        if seq_reset.dtype != torch.uint8 or tuple(seq_reset.shape) != (Bt, L) or not seq_reset.is_cuda or not seq_reset.is_contiguous():
            raise TypeError("seq_reset must be a contiguous uint8 device tensor [Bt, L]")
    return ssd_shape_t(dt, H, P, G, N, chunk, Bt, L, segment, 0, 0, 0, _ptr(seq_reset))


def ssd_workspace_bytes(shape: ssd_shape_t, is_backward: bool, flags: int = 0) -> int:
    return int(lib().ssd_workspace_bytes_flags(ctypes.byref(shape), 1 if is_backward else 0, flags))


def _check_inputs(x, dt, A, Bm, Cm, D, *more):
    import torch
    for t in (x, dt, Bm, Cm) + tuple(m for m in more if m is not None):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("tensors must be contiguous device tensors")
    for t in (dt, Bm, Cm):
        if t.dtype != x.dtype:
            raise TypeError("x, dt, B, C must share one storage dtype")
    for t in (A, D):
        if t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous():
            raise TypeError("A and D must be contiguous fp32 device tensors")


def _check_boundary(bnd, flags):
    import torch
    want = torch.bfloat16 if flags & SSD_FLAG_BF16_CHECKPOINTS else torch.float32
    if bnd is not None and bnd.dtype != want:
        raise TypeError(f"boundary_states must be {want} for these flags")


def _workspace(nbytes: int, device):
    import torch
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def ssd_fwd(x, dt, A, B, C, D, chunk, segment=None, init_state=None, flags=0, workspace=None, want_final=True,
            out=None, want_boundary=True, seq_reset=None):
    """y, final_state, boundary_states = ssd_fwd(...).  boundary_states is None when segment is None/L,
    or with want_boundary=False (forward only: no checkpoint is kept).
    `out` may carry preallocated tensors under the keys y, final_state, boundary_states."""
    import torch
    _check_inputs(x, dt, A, B, C, D, init_state)
    shape = make_shape(x, B, chunk, segment, seq_reset)
    Bt, L, H, P = x.shape
    N = B.shape[3]
    out = out or {}
    y = out["y"] if "y" in out else torch.empty_like(x)
    final = out.get("final_state")
    if final is None and want_final:
        final = torch.empty((Bt, H, P, N), dtype=torch.float32, device=x.device)
    nseg = -(-L // shape.segment) if L > 0 and shape.segment > 0 else 1
    bnd = out.get("boundary_states")
    if bnd is None and segment is not None and want_boundary:
        ck = torch.bfloat16 if flags & SSD_FLAG_BF16_CHECKPOINTS else torch.float32
        bnd = torch.empty((Bt, nseg, H, P, N), dtype=ck, device=x.device)
    _check_boundary(bnd, flags)
    need = ssd_workspace_bytes(shape, False, flags)
    if workspace is None:
        workspace = _workspace(need, x.device)
    rc = lib().ssd_fwd(ctypes.byref(shape), _ptr(x), _ptr(dt), _ptr(A), _ptr(B), _ptr(C), _ptr(D), _ptr(init_state),
                       _ptr(y), _ptr(final), _ptr(bnd), _ptr(workspace), workspace.numel(), flags, _stream(x))
    if rc != 0:
        raise SSDError(rc, "ssd_fwd")
    return y, final, bnd


def ssd_init() -> None:
    rc = lib().ssd_init()
    if rc != 0:
        raise SSDError(rc, "ssd_init")


def ssd_fwd_static_bytes(shape: ssd_shape_t, flags: int = 0) -> int:
    return int(lib().ssd_fwd_static_bytes(ctypes.byref(shape), flags))


def ssd_fwd_static(x, dt, A, B, C, D, chunk, segment, out, init_state=None, flags=0, seq_reset=None):
    """ssd_fwd without a workspace (the library's own device array): `out` must carry the preallocated
    tensors y and, optionally, final_state and boundary_states; nothing is allocated here or in the library."""
    _check_inputs(x, dt, A, B, C, D, init_state)
    shape = make_shape(x, B, chunk, segment, seq_reset)
    bnd = out.get("boundary_states")
    _check_boundary(bnd, flags)
    rc = lib().ssd_fwd_static(ctypes.byref(shape), _ptr(x), _ptr(dt), _ptr(A), _ptr(B), _ptr(C), _ptr(D), _ptr(init_state),
                              _ptr(out["y"]), _ptr(out.get("final_state")), _ptr(bnd), flags, _stream(x))
    if rc != 0:
        raise SSDError(rc, "ssd_fwd_static")
    return out["y"], out.get("final_state"), bnd


def ssd_decode(x, dt, A, B, C, D, state, flags=0, out=None, seq_reset=None):
    """y = ssd_decode(...): the recurrence token by token over x's T tokens; `state` [Bt,H,P,N] fp32 is
    updated in place."""
    import torch
    _check_inputs(x, dt, A, B, C, D, state)
    if state.dtype != torch.float32:
        raise TypeError("state must be fp32")
    shape = make_shape(x, B, 1, None, seq_reset)
    y = out if out is not None else torch.empty_like(x)
    rc = lib().ssd_decode(ctypes.byref(shape), _ptr(x), _ptr(dt), _ptr(A), _ptr(B), _ptr(C), _ptr(D), _ptr(state),
                          _ptr(y), flags, _stream(x))
    if rc != 0:
        raise SSDError(rc, "ssd_decode")
    return y


def _conv_shape(u):
    import torch
    Bt, L, C = u.shape
    if u.dtype == torch.bfloat16:
        dt = SSD_BF16
    elif u.dtype == torch.float32:
        dt = SSD_F32
    else:
        raise TypeError(f"unsupported dtype {u.dtype}")
    return ssd_conv_shape_t(dt, C, Bt, L, 0, 0)


def _conv_check(u, w, bias, *more):
    import torch
    for t in (u,) + tuple(m for m in more if m is not None):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("tensors must be contiguous device tensors")
    for t in (w, bias):
        if t is not None and (t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous()):
            raise TypeError("w and bias must be contiguous fp32 device tensors")


def ssd_conv1d_fwd(u, w, bias=None, state_in=None, want_state=True):
    """out, state_out = causal depthwise conv (kernel 4) + bias + SiLU of u [Bt,L,C] from state_in [Bt,3,C]."""
    import torch
    _conv_check(u, w, bias, state_in)
    shape = _conv_shape(u)
    out = torch.empty_like(u)
    state_out = torch.empty((u.shape[0], 3, u.shape[2]), dtype=u.dtype, device=u.device) if want_state else None
    rc = lib().ssd_conv1d_fwd(ctypes.byref(shape), _ptr(u), _ptr(w), _ptr(bias), _ptr(state_in), _ptr(out),
                              _ptr(state_out), _stream(u))
    if rc != 0:
        raise SSDError(rc, "ssd_conv1d_fwd")
    return out, state_out


def ssd_conv1d_bwd(u, w, bias, state_in, dout, dstate_out=None, want_dstate=True, flags=0, dw=None, dbias=None):
    """dict(du, dw, dbias, dstate_in) for the loss <dout, out> + <dstate_out, state_out>."""
    import torch
    _conv_check(u, w, bias, state_in, dout, dstate_out)
    shape = _conv_shape(u)
    Bt, L, C = u.shape
    du = torch.empty_like(u)
    if dw is None:
        dw = torch.empty((C, 4), dtype=torch.float32, device=u.device)
    if dbias is None and bias is not None:
        dbias = torch.empty((C,), dtype=torch.float32, device=u.device)
    dstate_in = torch.empty((Bt, 3, C), dtype=torch.float32, device=u.device) if want_dstate else None
    ws = _workspace(int(lib().ssd_conv1d_workspace_bytes(ctypes.byref(shape))), u.device)
    rc = lib().ssd_conv1d_bwd(ctypes.byref(shape), _ptr(u), _ptr(w), _ptr(bias), _ptr(state_in), _ptr(dout),
                              _ptr(dstate_out), _ptr(du), _ptr(dw), _ptr(dbias), _ptr(dstate_in), _ptr(ws), ws.numel(),
                              flags, _stream(u))
    if rc != 0:
        raise SSDError(rc, "ssd_conv1d_bwd")
    return {"du": du, "dw": dw, "dbias": dbias, "dstate_in": dstate_in}


def _norm_shape(y, z, ngroups, eps, *same_as):
    """y, z: [rows, dim] with unit stride along dim (rows may be a column slice of a wider tensor)."""
    import torch
    for t in (y,) if z is None else (y, z):
        if t.dim() != 2 or not t.is_cuda or (t.shape[1] > 1 and t.stride(1) != 1) or t.shape != y.shape or t.dtype != y.dtype:
            raise ValueError("y and z must be [rows, dim] device tensors of one dtype with unit stride along dim")
    for t, like in same_as:
        if t.shape != like.shape or t.stride() != like.stride() or t.dtype != like.dtype or not t.is_cuda:
            raise ValueError("gradient tensors must match the layout of what they are gradients of")
    dt = SSD_BF16 if y.dtype == torch.bfloat16 else SSD_F32
    if dt == SSD_F32 and y.dtype != torch.float32:
        raise TypeError("dtype must be float32 or bfloat16")
    T, C = y.shape
    return ssd_norm_shape_t(dt, C, ngroups, eps, T, y.stride(0) if T > 1 else C, z.stride(0) if z is not None and T > 1 else C)


def _norm_weight(w, C):
    import torch
    if w.dtype != torch.float32 or not w.is_cuda or not w.is_contiguous() or w.numel() != C:
        raise TypeError("w must be a contiguous fp32 device tensor of dim elements")


def ssd_gated_norm_fwd(y, z, w, eps=1e-5, ngroups=1):
    """out = RMSNorm_groups(y * silu(z)) * w for y, z [rows, dim]; out is dense.  z=None: no gate."""
    import torch
    shape = _norm_shape(y, z, ngroups, eps)
    _norm_weight(w, y.shape[1])
    out = torch.empty(y.shape, dtype=y.dtype, device=y.device)
    rc = lib().ssd_gated_norm_fwd(ctypes.byref(shape), _ptr(y), _ptr(z), _ptr(w), _ptr(out), _stream(y))
    if rc != 0:
        raise SSDError(rc, "ssd_gated_norm_fwd")
    return out


def ssd_gated_norm_bwd(y, z, w, dout, eps=1e-5, ngroups=1, flags=0, dy=None, dz=None, dw=None):
    """dict(dy, dz, dw) for the loss <dout, out>.  dy / dz may be given (laid out as y / z, e.g. column slices).
    z=None: no gate, dz stays None."""
    import torch
    if dy is None:
        dy = torch.empty_strided(y.shape, y.stride(), dtype=y.dtype, device=y.device)
    if z is None:
        if dz is not None:
            raise ValueError("dz without z")
        shape = _norm_shape(y, None, ngroups, eps, (dy, y))
    else:
        if dz is None:
            dz = torch.empty_strided(z.shape, z.stride(), dtype=z.dtype, device=z.device)
        shape = _norm_shape(y, z, ngroups, eps, (dy, y), (dz, z))
    _norm_weight(w, y.shape[1])
    if not dout.is_cuda or not dout.is_contiguous() or dout.shape != y.shape or dout.dtype != y.dtype:
        raise ValueError("dout must be a dense [rows, dim] device tensor of y's dtype")
    if dw is None:
        dw = torch.empty((y.shape[1],), dtype=torch.float32, device=y.device)
    ws = _workspace(int(lib().ssd_gated_norm_workspace_bytes(ctypes.byref(shape))), y.device)
    rc = lib().ssd_gated_norm_bwd(ctypes.byref(shape), _ptr(y), _ptr(z), _ptr(w), _ptr(dout), _ptr(dy), _ptr(dz), _ptr(dw),
                                  _ptr(ws), ws.numel(), flags, _stream(y))
    if rc != 0:
        raise SSDError(rc, "ssd_gated_norm_bwd")
    return {"dy": dy, "dz": dz, "dw": dw}


def _rows_view(t, name):
    import torch
    if t.dim() != 2 or not t.is_cuda or t.dtype != torch.bfloat16 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError(f"{name} must be a [rows, dim] bf16 device tensor with unit stride along dim")
    return t.stride(0) if t.shape[0] > 1 else t.shape[1]


def ssd_linear_fwd(x, w, out=None):
    """out [rows, out_dim] = x [rows, in_dim] @ w[out_dim, in_dim]^T (bf16, fp32 accumulation)."""
    import torch
    ldx = _rows_view(x, "x")
    if w.dim() != 2 or not w.is_cuda or w.dtype != torch.bfloat16 or not w.is_contiguous() or w.shape[1] != x.shape[1]:
        raise ValueError("w must be a dense [out_dim, in_dim] bf16 device tensor")
    if out is None:
        out = torch.empty((x.shape[0], w.shape[0]), dtype=torch.bfloat16, device=x.device)
    ldo = _rows_view(out, "out")
    if out.shape != (x.shape[0], w.shape[0]):
        raise ValueError("out must be [rows, out_dim]")
    rc = lib().ssd_linear_fwd(x.shape[0], x.shape[1], w.shape[0], _ptr(x), ldx, _ptr(w), _ptr(out), ldo, _stream(x))
    if rc != 0:
        raise SSDError(rc, "ssd_linear_fwd")
    return out


def ssd_linear_bwd(x, w, dout, want_dx=True, want_dw=True, flags=0, dx=None, dw=None):
    """dict(dx, dw) for the loss <dout, out>; dw is fp32 [out_dim, in_dim]."""
    import torch
    ldx = _rows_view(x, "x")
    ldd = _rows_view(dout, "dout")
    rows, in_dim = x.shape
    out_dim = w.shape[0]
    if w.dtype != torch.bfloat16 or not w.is_contiguous() or w.shape != (out_dim, in_dim) or dout.shape != (rows, out_dim):
        raise ValueError("w must be dense bf16 [out_dim, in_dim] and dout [rows, out_dim]")
    if dx is None and want_dx:
        dx = torch.empty((rows, in_dim), dtype=torch.bfloat16, device=x.device)
    lddx = _rows_view(dx, "dx") if dx is not None else 0
    if dw is None and want_dw:
        dw = torch.empty((out_dim, in_dim), dtype=torch.float32, device=x.device)
    if dw is not None and (dw.dtype != torch.float32 or not dw.is_contiguous() or dw.shape != (out_dim, in_dim)):
        raise ValueError("dw must be a dense fp32 [out_dim, in_dim] device tensor")
    rc = lib().ssd_linear_bwd(rows, in_dim, out_dim, _ptr(x), ldx, _ptr(w), _ptr(dout), ldd, _ptr(dx), lddx, _ptr(dw), flags,
                              _stream(x))
    if rc != 0:
        raise SSDError(rc, "ssd_linear_bwd")
    return {"dx": dx, "dw": dw}


def _block_setup(u, params, nheads, headdim, ngroups, dstate, chunk, segment, eps):
    import torch
    if u.dim() != 2 or u.dtype != torch.bfloat16 or not u.is_cuda or not u.is_contiguous():
        raise ValueError("u must be a dense [L, d_model] bf16 device tensor")
    L, dm = u.shape
    d_inner, gn = nheads * headdim, ngroups * dstate
    conv_dim, d_in_proj = d_inner + 2 * gn, 2 * d_inner + 2 * gn + nheads
    want = {"W_in": ((d_in_proj, dm), torch.bfloat16), "conv_w": ((conv_dim, 4), torch.float32), "conv_b": ((conv_dim,), torch.float32),
            "dt_bias": ((nheads,), torch.float32), "A": ((nheads,), torch.float32), "D": ((nheads,), torch.float32),
            "norm_w": ((d_inner,), torch.float32), "W_out": ((dm, d_inner), torch.bfloat16)}
    if params.get("pre_norm_w") is not None:
        want["pre_norm_w"] = ((dm,), torch.float32)
    for k, (shp, dty) in want.items():
        t = params[k]
        if tuple(t.shape) != shp or t.dtype != dty or not t.is_cuda or not t.is_contiguous():
            raise ValueError(f"params[{k!r}] must be a dense {dty} device tensor of shape {shp}")
    seg = segment if segment is not None else max(chunk, -(-L // chunk) * chunk)
    shape = magc_block_shape_t(dm, nheads, headdim, ngroups, dstate, chunk, eps, L, seg)
    par = magc_block_params_t(*[_ptr(params.get(k)) for k in BLOCK_PARAMS])
    nseg = max(1, -(-L // seg))
    return shape, par, want, nseg, conv_dim


def _block_states(init_ssm, init_conv, nheads, headdim, dstate, conv_dim, conv_dtype):
    import torch
    for t, shp, dty in ((init_ssm, (nheads, headdim, dstate), torch.float32), (init_conv, (3, conv_dim), conv_dtype)):
        if t is not None and (tuple(t.shape) != shp or t.dtype != dty or not t.is_cuda or not t.is_contiguous()):
            raise ValueError(f"state tensor must be a dense {dty} device tensor of shape {shp}")


def magc_block_fwd(u, params, nheads, headdim, ngroups, dstate, chunk, segment=None, eps=1e-5, init_ssm=None, init_conv=None,
                   checkpoints=True):
    """One Mamba-2 block over u [L, d_model] from the states (init_ssm, init_conv) (None = zeros), with sequence
    checkpoints every `segment` tokens, or none at all (checkpoints=False: prefill / generation).
    Returns dict(out, ssm_ckpt, conv_ckpt, final_ssm, final_conv)."""
    import torch
    shape, par, _, nseg, conv_dim = _block_setup(u, params, nheads, headdim, ngroups, dstate, chunk, segment, eps)
    _block_states(init_ssm, init_conv, nheads, headdim, dstate, conv_dim, torch.bfloat16)
    dev = u.device
    out = torch.empty_like(u)
    ssm_ckpt = torch.zeros((nseg, nheads, headdim, dstate), dtype=torch.float32, device=dev) if checkpoints else None
    conv_ckpt = torch.zeros((nseg, 3, conv_dim), dtype=torch.bfloat16, device=dev) if checkpoints else None
    final_ssm = torch.empty((nheads, headdim, dstate), dtype=torch.float32, device=dev)
    final_conv = torch.empty((3, conv_dim), dtype=torch.bfloat16, device=dev)
    ws = _workspace(int(lib().magc_block_workspace_bytes(ctypes.byref(shape), 0)), dev)
    rc = lib().magc_block_fwd(ctypes.byref(shape), ctypes.byref(par), _ptr(u), _ptr(init_ssm), _ptr(init_conv), _ptr(out),
                              _ptr(ssm_ckpt), _ptr(conv_ckpt), _ptr(final_ssm), _ptr(final_conv), _ptr(ws), ws.numel(), _stream(u))
    if rc != 0:
        raise SSDError(rc, "magc_block_fwd")
    return {"out": out, "ssm_ckpt": ssm_ckpt, "conv_ckpt": conv_ckpt, "final_ssm": final_ssm, "final_conv": final_conv}


def magc_block_bwd(u, params, dout, ssm_ckpt, conv_ckpt, nheads, headdim, ngroups, dstate, chunk, segment=None, eps=1e-5,
                   flags=0, grads=None, init_ssm=None, init_conv=None, dfinal_ssm=None, dfinal_conv=None, want_dinit=False):
    """dict(du, dW_in, dconv_w, dconv_b, ddt_bias, dA, dD, dnorm_w, dW_out[, dpre_norm_w][, dinit_ssm, dinit_conv]) for the loss
    <dout, out> + <dfinal_ssm, final_ssm> + <dfinal_conv, final_conv>."""
    import torch
    shape, par, want, nseg, conv_dim = _block_setup(u, params, nheads, headdim, ngroups, dstate, chunk, segment, eps)
    _block_states(init_ssm, init_conv, nheads, headdim, dstate, conv_dim, torch.bfloat16)
    _block_states(dfinal_ssm, dfinal_conv, nheads, headdim, dstate, conv_dim, torch.float32)
    if dout.shape != u.shape or dout.dtype != u.dtype or not dout.is_cuda or not dout.is_contiguous():
        raise ValueError("dout must match u")
    dev = u.device
    if grads is None:
        grads = {"d" + k: torch.empty(shp, dtype=torch.float32, device=dev) for k, (shp, _) in want.items()}
    for k, (shp, _) in want.items():
        t = grads.get("d" + k)
        if t is None:   # the library refuses a missing one
            continue
        if tuple(t.shape) != shp or t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous():
            raise ValueError(f"grads['d{k}'] must be a dense fp32 device tensor of shape {shp}")
    gr = magc_block_grads_t(*[_ptr(grads.get("d" + k)) for k in BLOCK_PARAMS])
    du = torch.empty_like(u)
    dinit_ssm = torch.empty((nheads, headdim, dstate), dtype=torch.float32, device=dev) if want_dinit else None
    dinit_conv = torch.empty((3, conv_dim), dtype=torch.float32, device=dev) if want_dinit else None
    ws = _workspace(int(lib().magc_block_workspace_bytes(ctypes.byref(shape), 1)), dev)
    rc = lib().magc_block_bwd(ctypes.byref(shape), ctypes.byref(par), _ptr(u), _ptr(init_ssm), _ptr(init_conv), _ptr(dout),
                              _ptr(dfinal_ssm), _ptr(dfinal_conv), _ptr(ssm_ckpt), _ptr(conv_ckpt), _ptr(du), ctypes.byref(gr),
                              _ptr(dinit_ssm), _ptr(dinit_conv), _ptr(ws), ws.numel(), flags, _stream(u))
    if rc != 0:
        raise SSDError(rc, "magc_block_bwd")
    res = {"du": du, **grads}
    if want_dinit:
        res.update(dinit_ssm=dinit_ssm, dinit_conv=dinit_conv)
    return res


def _blockstack_setup(x0, layers, nheads, headdim, ngroups, dstate, chunk, segment, layer_interval, eps):
    shape, _, want, nseg, conv_dim = _block_setup(x0, layers[0], nheads, headdim, ngroups, dstate, chunk, segment, eps)
    for p in layers[1:]:
        _block_setup(x0, p, nheads, headdim, ngroups, dstate, chunk, segment, eps)
    if any((p.get("pre_norm_w") is None) != (layers[0].get("pre_norm_w") is None) for p in layers):
        raise ValueError("either every layer has pre_norm_w or none")
    pars = (magc_block_params_t * len(layers))(*[magc_block_params_t(*[_ptr(p.get(k)) for k in BLOCK_PARAMS]) for p in layers])
    sshape = magc_blockstack_shape_t(shape, len(layers), layer_interval)
    return sshape, pars, want, nseg, conv_dim


def magc_blockstack_fwd(x0, layers, nheads, headdim, ngroups, dstate, chunk, segment, layer_interval, eps=1e-5):
    """Residual stack of whole blocks (layers: list of parameter dicts) on the two-axis checkpoint grid.
    Returns dict(out, l_ckpt, ssm_ckpt, conv_ckpt)."""
    import torch
    sshape, pars, _, nseg, conv_dim = _blockstack_setup(x0, layers, nheads, headdim, ngroups, dstate, chunk, segment, layer_interval, eps)
    dev, (L, dm), NL = x0.device, x0.shape, len(layers)
    ngl = -(-NL // layer_interval)
    out = torch.empty_like(x0)
    l_ckpt = torch.empty((max(ngl - 1, 1), L, dm), dtype=torch.bfloat16, device=dev)
    ssm_ckpt = torch.zeros((NL, nseg, nheads, headdim, dstate), dtype=torch.float32, device=dev)
    conv_ckpt = torch.zeros((NL, nseg, 3, conv_dim), dtype=torch.bfloat16, device=dev)
    ws = _workspace(int(lib().magc_blockstack_workspace_bytes(ctypes.byref(sshape), 0)), dev)
    rc = lib().magc_blockstack_fwd(ctypes.byref(sshape), pars, _ptr(x0), _ptr(out), _ptr(l_ckpt), _ptr(ssm_ckpt), _ptr(conv_ckpt),
                                   _ptr(ws), ws.numel(), _stream(x0))
    if rc != 0:
        raise SSDError(rc, "magc_blockstack_fwd")
    return {"out": out, "l_ckpt": l_ckpt, "ssm_ckpt": ssm_ckpt, "conv_ckpt": conv_ckpt}


def magc_blockstack_infer(x0, layers, nheads, headdim, ngroups, dstate, chunk, segment, eps=1e-5, ssm_state=None, conv_state=None,
                          out=None, workspace=None):
    """The stack forward only with nothing kept, continuing from the per-layer states (None: a new sequence;
    then they are allocated).  The states are updated in place.  Returns dict(out, ssm_state, conv_state, workspace);
    hand the last three back in to continue the sequence without any allocation."""
    import torch
    sshape, pars, _, _, conv_dim = _blockstack_setup(x0, layers, nheads, headdim, ngroups, dstate, chunk, segment, 1, eps)
    dev, NL = x0.device, len(layers)
    if (ssm_state is None) != (conv_state is None):
        raise ValueError("both states or none")
    fresh = ssm_state is None
    if fresh:
        ssm_state = torch.empty((NL, nheads, headdim, dstate), dtype=torch.float32, device=dev)
        conv_state = torch.empty((NL, 3, conv_dim), dtype=torch.bfloat16, device=dev)
    for t, shp, dty in ((ssm_state, (NL, nheads, headdim, dstate), torch.float32), (conv_state, (NL, 3, conv_dim), torch.bfloat16)):
        if tuple(t.shape) != shp or t.dtype != dty or not t.is_cuda or not t.is_contiguous():
            raise ValueError(f"state tensor must be a dense {dty} device tensor of shape {shp}")
    if out is None:
        out = torch.empty_like(x0)
    elif out.shape != x0.shape or out.dtype != x0.dtype or not out.is_cuda or not out.is_contiguous():
        raise ValueError("out must match x0")
    need = int(lib().magc_blockstack_workspace_bytes(ctypes.byref(sshape), 0))
    if workspace is None or workspace.numel() < need:
        workspace = _workspace(need, dev)
    rc = lib().magc_blockstack_infer(ctypes.byref(sshape), pars, _ptr(x0), _ptr(out), _ptr(ssm_state), _ptr(conv_state), 1 if fresh else 0,
                                     _ptr(workspace), workspace.numel(), _stream(x0))
    if rc != 0:
        raise SSDError(rc, "magc_blockstack_infer")
    return {"out": out, "ssm_state": ssm_state, "conv_state": conv_state, "workspace": workspace}


def magc_blockstack_decode(x, layers, nheads, headdim, ngroups, dstate, chunk, segment, ssm_state, conv_state, eps=1e-5, out=None,
                           workspace=None):
    """One token for each of x.shape[0] <= 16 independent sequences: x [nseq, d_model]; ssm_state [nseq, NL, H, P, N] fp32
    and conv_state [nseq, NL, 3, conv_dim] bf16 are updated in place.  Returns dict(out, workspace)."""
    import torch
    sshape, pars, _, _, conv_dim = _blockstack_setup(x, layers, nheads, headdim, ngroups, dstate, chunk, segment, 1, eps)
    sshape.block.seqlen = 1      # a token per sequence: the shape the workspace is sized for
    dev, NL, nseq = x.device, len(layers), x.shape[0]
    for t, shp, dty in ((ssm_state, (nseq, NL, nheads, headdim, dstate), torch.float32), (conv_state, (nseq, NL, 3, conv_dim), torch.bfloat16)):
        if tuple(t.shape) != shp or t.dtype != dty or not t.is_cuda or not t.is_contiguous():
            raise ValueError(f"state tensor must be a dense {dty} device tensor of shape {shp}")
    if out is None:
        out = torch.empty_like(x)
    elif out.shape != x.shape or out.dtype != x.dtype or not out.is_cuda or not out.is_contiguous():
        raise ValueError("out must match x")
    need = int(lib().magc_blockstack_workspace_bytes(ctypes.byref(sshape), 0))
    if workspace is None or workspace.numel() < need:
        workspace = _workspace(need, dev)
    rc = lib().magc_blockstack_decode(ctypes.byref(sshape), pars, nseq, _ptr(x), _ptr(out), _ptr(ssm_state), _ptr(conv_state),
                                      _ptr(workspace), workspace.numel(), _stream(x))
    if rc != 0:
        raise SSDError(rc, "magc_blockstack_decode")
    return {"out": out, "workspace": workspace}


def magc_blockstack_bwd(x0, layers, dout, l_ckpt, ssm_ckpt, conv_ckpt, nheads, headdim, ngroups, dstate, chunk, segment,
                        layer_interval, eps=1e-5, flags=0, grads=None):
    """dict(dx0, grads=[per-layer dict of dW_in, dconv_w, dconv_b, ddt_bias, dA, dD, dnorm_w, dW_out])."""
    import torch
    sshape, pars, want, _, _ = _blockstack_setup(x0, layers, nheads, headdim, ngroups, dstate, chunk, segment, layer_interval, eps)
    dev = x0.device
    if grads is None:
        grads = [{"d" + k: torch.empty(shp, dtype=torch.float32, device=dev) for k, (shp, _) in want.items()} for _ in layers]
    for g in grads:
        for k, (shp, _) in want.items():
            t = g.get("d" + k)
            if t is None:
                continue
            if tuple(t.shape) != shp or t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous():
                raise ValueError(f"grads['d{k}'] must be a dense fp32 device tensor of shape {shp}")
    grs = (magc_block_grads_t * len(layers))(*[magc_block_grads_t(*[_ptr(g.get("d" + k)) for k in BLOCK_PARAMS]) for g in grads])
    if dout.shape != x0.shape or dout.dtype != x0.dtype or not dout.is_cuda or not dout.is_contiguous():
        raise ValueError("dout must match x0")
    dx0 = torch.empty_like(x0)
    ws = _workspace(int(lib().magc_blockstack_workspace_bytes(ctypes.byref(sshape), 1)), dev)
    rc = lib().magc_blockstack_bwd(ctypes.byref(sshape), pars, _ptr(x0), _ptr(dout), _ptr(l_ckpt), _ptr(ssm_ckpt), _ptr(conv_ckpt),
                                   _ptr(dx0), grs, _ptr(ws), ws.numel(), flags, _stream(x0))
    if rc != 0:
        raise SSDError(rc, "magc_blockstack_bwd")
    return {"dx0": dx0, "grads": grads}


def ssd_bwd(x, dt, A, B, C, D, dy, chunk, segment=None, init_state=None, dfinal_state=None, boundary_states=None,
            flags=0, workspace=None, dA=None, dD=None, want_dinit=True, out=None, seq_reset=None):
    """Returns dict(dx, ddt, dA, dB, dC, dD, dinit_state).  `out` may carry preallocated dx, ddt, dB, dC,
    dinit_state."""
    import torch
    _check_inputs(x, dt, A, B, C, D, dy, init_state, dfinal_state, boundary_states)
    shape = make_shape(x, B, chunk, segment, seq_reset)
    Bt, L, H, P = x.shape
    N = B.shape[3]
    out = out or {}
    dx = out["dx"] if "dx" in out else torch.empty_like(x)
    ddt = out["ddt"] if "ddt" in out else torch.empty_like(dt)
    dB = out["dB"] if "dB" in out else torch.empty_like(B)
    dC = out["dC"] if "dC" in out else torch.empty_like(C)
    if dA is None:
        dA = torch.empty((H,), dtype=torch.float32, device=x.device)
    if dD is None:
        dD = torch.empty((H,), dtype=torch.float32, device=x.device)
    dinit = out.get("dinit_state")
    if dinit is None and want_dinit:
        dinit = torch.empty((Bt, H, P, N), dtype=torch.float32, device=x.device)
    _check_boundary(boundary_states, flags)
    need = ssd_workspace_bytes(shape, True, flags)
    if workspace is None:
        workspace = _workspace(need, x.device)
    rc = lib().ssd_bwd(ctypes.byref(shape), _ptr(x), _ptr(dt), _ptr(A), _ptr(B), _ptr(C), _ptr(D), _ptr(init_state),
                       _ptr(dy), _ptr(dfinal_state), _ptr(boundary_states), _ptr(dx), _ptr(ddt), _ptr(dA), _ptr(dB),
                       _ptr(dC), _ptr(dD), _ptr(dinit), _ptr(workspace), workspace.numel(), flags, _stream(x))
    if rc != 0:
        raise SSDError(rc, "ssd_bwd")
    return {"dx": dx, "ddt": ddt, "dA": dA, "dB": dB, "dC": dC, "dD": dD, "dinit_state": dinit}


def magc_stack_workspace_bytes(shape: ssd_shape_t, nlayers: int, layer_interval: int, is_backward: bool) -> int:
    return int(lib().magc_stack_workspace_bytes(ctypes.byref(shape), nlayers, layer_interval, 1 if is_backward else 0))


def magc_stack_fwd(x0, dt, A, B, C, D, chunk, segment, layer_interval, workspace=None, want_final=True):
    """dt [nl,Bt,L,H], A/D [nl,H], B/C [nl,Bt,L,G,N].  Returns dict(out, final_states, s_ckpt, l_ckpt)."""
    import torch
    nl = dt.shape[0]
    _check_inputs(x0, dt, A, B[0], C[0], D)
    shape = make_shape(x0, B[0], chunk, segment)
    Bt, L, H, P = x0.shape
    N = B.shape[4]
    nseg = L // segment
    l = min(layer_interval, nl)
    nlg = (nl + l - 1) // l
    out = torch.empty_like(x0)
    finals = torch.empty((nl, Bt, H, P, N), dtype=torch.float32, device=x0.device) if want_final else None
    s_ckpt = torch.empty((nl, Bt, nseg, H, P, N), dtype=torch.float32, device=x0.device)
    l_ckpt = torch.empty((nlg - 1, Bt, L, H, P), dtype=x0.dtype, device=x0.device) if nlg > 1 else None
    if workspace is None:
        workspace = _workspace(magc_stack_workspace_bytes(shape, nl, layer_interval, False), x0.device)
    rc = lib().magc_stack_fwd(ctypes.byref(shape), nl, layer_interval, _ptr(x0), _ptr(dt), _ptr(A), _ptr(B), _ptr(C),
                              _ptr(D), _ptr(out), _ptr(finals), _ptr(s_ckpt), _ptr(l_ckpt), _ptr(workspace),
                              workspace.numel(), _stream(x0))
    if rc != 0:
        raise SSDError(rc, "magc_stack_fwd")
    return {"out": out, "final_states": finals, "s_ckpt": s_ckpt, "l_ckpt": l_ckpt}


def magc_stack_bwd(x0, dt, A, B, C, D, dout, s_ckpt, l_ckpt, chunk, segment, layer_interval, workspace=None):
    """Returns dict(dx0, ddt, dA, dB, dC, dD) with the per-layer gradients stacked like the inputs."""
    import torch
    nl = dt.shape[0]
    _check_inputs(x0, dt, A, B[0], C[0], D, dout, s_ckpt, l_ckpt)
    shape = make_shape(x0, B[0], chunk, segment)
    H = x0.shape[2]
    dx0 = torch.empty_like(x0)
    ddt = torch.empty_like(dt)
    dB = torch.empty_like(B)
    dC = torch.empty_like(C)
    dA = torch.empty((nl, H), dtype=torch.float32, device=x0.device)
    dD = torch.empty((nl, H), dtype=torch.float32, device=x0.device)
    if workspace is None:
        workspace = _workspace(magc_stack_workspace_bytes(shape, nl, layer_interval, True), x0.device)
    rc = lib().magc_stack_bwd(ctypes.byref(shape), nl, layer_interval, _ptr(x0), _ptr(dt), _ptr(A), _ptr(B), _ptr(C),
                              _ptr(D), _ptr(dout), _ptr(s_ckpt), _ptr(l_ckpt), _ptr(dx0), _ptr(ddt), _ptr(dA),
                              _ptr(dB), _ptr(dC), _ptr(dD), _ptr(workspace), workspace.numel(), _stream(x0))
    if rc != 0:
        raise SSDError(rc, "magc_stack_bwd")
    return {"dx0": dx0, "ddt": ddt, "dA": dA, "dB": dB, "dC": dC, "dD": dD}


def magc_plan(n_layers, seqlen, c_lckpt, c_sckpt, c_grid, c_state, s_multiple=256, budget=0.0, integer_counts=False):
    """Host-only planner.  Returns (status, dict).  status is 0 or SSD_ERR_BUDGET (-7) with the
    minimum-memory plan filled in; any other error raises."""
    m = magc_model_t(n_layers, seqlen, c_lckpt, c_sckpt, c_grid, c_state, s_multiple, budget, 1 if integer_counts else 0)
    p = magc_plan_t()
    rc = lib().magc_plan(ctypes.byref(m), ctypes.byref(p))
    if rc not in (0, -7):
        raise SSDError(rc, "magc_plan")
    return rc, {"l": p.l, "s": p.s, "m_lckpt": p.m_lckpt, "m_sckpt": p.m_sckpt, "m_grid": p.m_grid,
                "m_state": p.m_state, "m_total": p.m_total, "regime": p.regime, "fits": bool(p.fits)}


def ssd_prof_kernel_id(name: str) -> int:
    kid = 0
    while True:
        n = lib().ssd_prof_kernel_name(kid)
        if n is None:
            raise KeyError(name)
        if n.decode() == name:
            return kid
        kid += 1


def ssd_prof_enable(on, only: Optional[str] = None) -> None:
    """on: record every kernel launch; only=name: record launches of that kernel alone."""
    mode = (2 + ssd_prof_kernel_id(only)) if (on and only is not None) else (1 if on else 0)
    rc = lib().ssd_prof_enable(mode)
    if rc != 0:
        raise SSDError(rc, "ssd_prof_enable")


def ssd_prof_serialize(on: bool) -> None:
    """Keep every segment on the caller's stream (no overlap between kernels) while `on`."""
    lib().ssd_prof_serialize(1 if on else 0)


def ssd_prof_read() -> dict:
    """{kernel name: (total milliseconds, launches)} for every kernel launched since ssd_prof_enable(True)."""
    out = {}
    kid = 0
    while True:
        name = lib().ssd_prof_kernel_name(kid)
        if name is None:
            break
        ms, n = ctypes.c_double(0.0), ctypes.c_int64(0)
        rc = lib().ssd_prof_read(kid, ctypes.byref(ms), ctypes.byref(n))
        if rc != 0:
            raise SSDError(rc, "ssd_prof_read")
        if n.value:
            out[name.decode()] = (ms.value, n.value)
        kid += 1
    return out
