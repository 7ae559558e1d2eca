"""MI355X (gfx950) integer-only inference kernels for HAWQ-V3: thin Python binding over the
C interface declared in ``include/hawq.h``.  Every step of the path runs in the HIP library;
this package only marshals arguments (PyTorch supplies device memory and streams)."""
from .binding import (  # noqa: F401
    U8, S8, U4, S4, S32, HawqError, load_library, status_string,
    hawq_conv2d_int, hawq_conv2d_dual_int, hawq_gemm_int, hawq_residual_add_dyadic, hawq_avgpool_int, hawq_maxpool_int,
    hawq_pool2d_sum_int, hawq_concat_dyadic,
    hawq_net_num_layers, hawq_net_layer_info, hawq_tune_set_tile, hawq_tune_set_split, hawq_tune_set_fusion, hawq_probe_mfma_peak, hawq_conv_blocked_weights_bytes, hawq_conv_block_weights, hawq_noalloc_workspace_limit, hawq_conv_fragment_weights_bytes, hawq_conv_fragment_weights,
    hawq_bottleneck_tail_int, HawqNet, ConvDesc,
)
