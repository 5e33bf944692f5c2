"""MI355X-native generalized-Gaussian tensor pass: thin Python binding over libgg (HIP, gfx950).

The binding only marshals arguments; every step of the pass runs in the library's kernels.
PyTorch supplies device memory and streams.  There is no CPU fallback: if the compiled library
is missing, importing `binding` symbols raises.
"""
from .binding import (  # noqa: F401
    GG_F32, GG_BF16, GG_FLOOR, GG_NEAREST_EVEN, GG_EG_TILE,
    GG_F_EMPTY, GG_F_DEGENERATE, GG_F_BETA_CLAMPED_LO, GG_F_BETA_CLAMPED_HI, GG_F_NONFINITE, GG_F_SATURATED,
    FIT_DTYPE, RATE_DTYPE, GGError, lib, lib_path, workspace_bytes, Workspace,
    gg_fit, gg_fit_segmented, gg_fit_rows, gg_quantize_rate, gg_quantize_rate_segmented, gg_quantize_rate_rows,
    gg_delta_from_fit, gg_penalty_grad, gg_penalty_grad_segmented, gg_sample, gg_philox_words, gg_init_alpha,
    gg_compression_ratio, gg_fused_segmented, gg_fused_segmented_noalloc, gg_fused_rows, fit_records, rate_records,
    gg_rate_grad, gg_gct_update, gg_gct_update_segmented, gg_eg_encode, gg_eg_encode_tensor, gg_eg_encode_segmented, gg_eg_decode, gg_eg_decode_dequant, gg_eg_decode_dequant_segmented, eg_buffers, gg_huffman_mean_bits,
)
from .train import gg_init_, eg_rate, EGRate, GCTState  # noqa: F401,E402
