"""MI355X-native quantized linear layer of ViDiT-Q (arxiv 2406.02540).

`binding` wraps the C-ABI library libvidiq.so (hand-written gfx950 kernels);
`workloads` draws the seeded synthetic DiT-shaped inputs; `build` compiles the library.
"""
from .binding import (  # noqa: F401
    VqError,
    vq_balance_mask,
    vq_channel_absmax,
    vq_gelu_linear,
    vq_gelu_quantize,
    vq_gemm_f16,
    vq_hadamard_linear,
    vq_hadamard_quantize,
    vq_gemm_w4a8,
    vq_gemm_w8a8,
    vq_layernorm_linear,
    vq_layernorm_quantize,
    vq_linear,
    vq_linear_static,
    vq_linear_workspace_bytes,
    vq_quantize_per_token,
    vq_quantize_static,
    vq_quantize_weight,
    vq_residual_linear,
    vq_residual_quantize,
    vq_rotate_weight,
)
