"""glowmi: the lowered Convolution / FullyConnected hot path of the Glow paper (arXiv 1805.00907)
as hand-written HIP kernels for AMD MI355X, behind a C ABI (include/glowmi.h).

This package is only the thin Python face of that library: it marshals torch device tensors into
the C calls.  Every step of the computation runs in the HIP kernels; there is no CPU fallback, and
loading fails loudly when the library has not been built (python -m paper_1805_00907_amd.build).
"""
from .binding import (  # noqa: F401
    ACT_NONE,
    ACT_RELU,
    Chain,
    ChainOp,
    ConvDesc,
    GlowmiError,
    QParam,
    SeqLayer,
    conv2d,
    conv2d_chain,
    conv2d_chainv,
    conv2d_chainv_workspace_bytes,
    conv2d_workspace_bytes,
    conv_out_shape,
    dequantize,
    fc,
    fc_noalloc,
    fc_noalloc_max_scratch_bytes,
    fc_workspace_bytes,
    fold_batchnorm,
    last_variant,
    library,
    library_path,
    qconv2d,
    qconv2d_chain,
    qconv2d_chainv,
    qconv2d_chainv_workspace_bytes,
    qconv2d_workspace_bytes,
    qfc,
    qfc_workspace_bytes,
    quantize,
    requant_params,
    rescale,
    rescale_params,
    seq_arena_bytes,
    seq_conv2d,
    seq_layers,
    seq_qconv2d,
    tuning_reset,
    tuning_set,
)
