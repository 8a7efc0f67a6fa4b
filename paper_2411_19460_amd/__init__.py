"""MI355X-native Mamba-2 SSD selective scan (forward + backward) with Multi-Axis Gradient
Checkpointing.  The work happens in libssd_magc.so (HIP, gfx950); `binding` marshals arguments,
`synth` draws the seeded benchmark inputs."""
from . import synth  # noqa: F401
from .binding import (SSD_BF16, SSD_F32, SSD_FLAG_ACCUM_PARAM, SSD_FLAG_BF16_CHECKPOINTS, SSD_FLAG_FP32_CHUNK_STATES, SSD_FLAG_GENERIC_KERNELS, SSD_FLAG_RESIDUAL,  # noqa: F401
                      SSDError, lib, magc_block_bwd, magc_block_fwd, magc_blockstack_bwd, magc_blockstack_fwd, magc_blockstack_decode, magc_blockstack_infer, magc_plan, magc_stack_bwd, magc_stack_fwd, magc_stack_workspace_bytes, make_shape,
                      ssd_bwd, ssd_conv1d_bwd, ssd_conv1d_fwd, ssd_conv_shape_t, ssd_decode, ssd_gated_norm_bwd, ssd_gated_norm_fwd, ssd_linear_bwd, ssd_linear_fwd, ssd_norm_shape_t, ssd_fwd, ssd_fwd_static, ssd_fwd_static_bytes, ssd_init, ssd_prof_enable, ssd_prof_read, ssd_prof_serialize, ssd_shape_t, ssd_workspace_bytes, strerror)


def __getattr__(name):
    # the autograd wrapper imports torch: load it on first use only
    if name == "ssd_scan":
        from .autograd import ssd_scan
        return ssd_scan
    raise AttributeError(name)
