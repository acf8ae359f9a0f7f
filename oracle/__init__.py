"""CPU fp64 oracle for Dynamic Mask Attention (arxiv 2508.02124).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this
package; only the test-suite, the smoke check and the benchmark's CPU-baseline
leg do.  It shares no code with the HIP path.
"""
from .dma_oracle import (  # noqa: F401
    softplus,
    z_scores,
    kept_mask_definition,
    kept_mask_ranked,
    expiry_from_kept,
    expiry_sequential,
    topk_indices,
    dma_forward,
    dma_backward,
    dma_forward_gather_loop,
    dma_scalar_bruteforce,
    n_active_pairs,
    dma_rows,
    dma_keys,
    mask_backward,
    dma_decode,
    z_scores_xhead,
    xhead_backward,
    expand_bias,
    bias_backward,
)
