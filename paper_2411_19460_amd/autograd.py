"""torch.autograd face of the C ABI: `ssd_scan(...)` is differentiable and keeps, between forward and
backward, only what MA-GC keeps (Sec. 3.2-3.3: the state entering every segment) -- the backward pass
calls ssd_bwd, which restores each segment from its checkpoint.  Argument marshalling only: every
step of the computation runs in libssd_magc.so."""
from __future__ import annotations

import torch

from . import binding


class _SSDScan(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, dt, A, B, C, D, init_state, chunk, segment, flags, seq_reset):
        y, final, bnd = binding.ssd_fwd(x, dt, A, B, C, D, chunk, segment, init_state, flags, seq_reset=seq_reset)
        ctx.save_for_backward(x, dt, A, B, C, D, init_state if init_state is not None else x.new_empty(0),
                              bnd if bnd is not None else x.new_empty(0))
        ctx.cfg = (chunk, segment, flags, init_state is not None, bnd is not None)
        ctx.seq_reset = seq_reset
        return y, final

    @staticmethod
    def backward(ctx, dy, dfinal):
        x, dt, A, B, C, D, init_state, bnd = ctx.saved_tensors
        chunk, segment, flags, has_init, has_bnd = ctx.cfg
        if dy is None:
            dy = torch.zeros_like(x)
        g = binding.ssd_bwd(x, dt, A, B, C, D, dy.contiguous(), chunk, segment, init_state if has_init else None,
                            dfinal.contiguous() if dfinal is not None else None, bnd if has_bnd else None, flags,
                            want_dinit=has_init and ctx.needs_input_grad[6], seq_reset=ctx.seq_reset)
        return (g["dx"], g["ddt"], g["dA"], g["dB"], g["dC"], g["dD"],
                g["dinit_state"] if has_init and ctx.needs_input_grad[6] else None, None, None, None, None)


def ssd_scan(x, dt, A, B, C, D, chunk, segment=None, init_state=None, flags=0, seq_reset=None):
    """y, final_state = ssd_scan(...): one SSD layer (Sec. 3.1, Eq. 1 in the Mamba-2 form), differentiable in
    x, dt, A, B, C, D and init_state.  `segment` is the checkpoint interval in tokens (None: the whole
    sequence is one segment).  seq_reset [Bt, L] uint8 marks the first token of every packed sequence.
    Tensors as in ssd_fwd (contiguous device tensors; dt already positive)."""
    return _SSDScan.apply(x, dt, A, B, C, D, init_state, chunk, segment, flags, seq_reset)
