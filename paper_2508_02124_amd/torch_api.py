"""torch.autograd glue over the C-ABI library: a differentiable function and a drop-in module.

Nothing here computes: tensors are allocated with torch, their addresses are handed to
dma_mask_gen / dma_fwd / dma_bwd / dma_mask_bwd, and the results are returned to autograd.
The paper names this integration as its own future work (Section 7); the operations are
those of Section 4: Eq. 3-6 forward, Eq. 7-10 backward, and the chain rule of Eq. 3 that
carries the bias gradient on to the score parameters (Section 6).

Layout: packed tokens, Q [T, H_q, d], K, V [T, H_kv, d] (bf16 or fp32, contiguous), W [H_q, d]
and A [H_q] fp32, cu_seqlens [n_docs + 1] int32 on the same device.  A W of shape
[H_q, H_kv * d] selects the paper's full cross-head sampling tensor (Eq. 3: the score of a head
contracts the token's values of all heads; dma_scores_xhead and its chain rule).  The selection of
the kept keys is piecewise constant, so no gradient flows through it (Section 6).
"""
from __future__ import annotations

import math

import torch

from . import binding as B


def _dtype_code(t):
    if t.dtype == torch.bfloat16:
        return B.DMA_BF16
    if t.dtype == torch.float32:
        return B.DMA_F32
    raise TypeError(f"Q/K/V must be bfloat16 or float32, got {t.dtype}")


def _check_inputs(Q, K, V, W, A, cu_seqlens):
    for name, t in (("Q", Q), ("K", K), ("V", V), ("W", W), ("A", A), ("cu_seqlens", cu_seqlens)):
        if not t.is_cuda:
            raise RuntimeError(f"{name} must live on the GPU: this library has no CPU path")
    if Q.dim() != 3 or K.dim() != 3 or K.shape != V.shape or Q.shape[0] != K.shape[0] or Q.shape[2] != K.shape[2]:
        raise ValueError("expected Q [T, H_q, d] and K, V [T, H_kv, d]")
    if K.dtype != Q.dtype or V.dtype != Q.dtype:
        raise TypeError("Q, K, V must share one dtype")
    H_q, d = Q.shape[1], Q.shape[2]
    if W.shape not in ((H_q, d), (H_q, K.shape[1] * d)) or A.shape != (H_q,):
        raise ValueError("expected W [H_q, d] (per head) or [H_q, H_kv * d] (cross-head) and A [H_q]")
    if W.dtype != torch.float32 or A.dtype != torch.float32 or cu_seqlens.dtype != torch.int32:
        raise TypeError("W, A must be float32 and cu_seqlens int32")


class DynamicMaskAttentionFunction(torch.autograd.Function):
    """O = DMA(Q, K, V; W, A) on packed variable-length documents; differentiable in Q, K, V, W, A."""

    @staticmethod
    def forward(ctx, Q, K, V, W, A, cu_seqlens, k, max_seqlen=0, softmax_scale=0.0, bias=None):
        _check_inputs(Q, K, V, W, A, cu_seqlens)
        Q, K, V, W, A = (t.contiguous() for t in (Q, K, V, W, A))
        T, H_q, d = Q.shape
        bias_heads, bias_per_token = 0, True
        if bias is not None:
            # one value per key, broadcast over the query rows: [H_q or 1, T] (packed like the tokens) or
            # [H_q or 1, max_seqlen] (by position in the document, shared by all documents)
            if (not bias.is_cuda or bias.dtype != torch.float32 or bias.dim() != 2 or bias.shape[0] not in (1, H_q)
                    or bias.shape[1] not in (T, max_seqlen)):
                raise ValueError("bias must be a float32 GPU tensor [H_q or 1, T] or [H_q or 1, max_seqlen]")
            bias = bias.contiguous()
            bias_heads, bias_per_token = bias.shape[0], bias.shape[1] == T
        shape = B.make_shape(T, cu_seqlens.numel() - 1, H_q, K.shape[1], d, k, causal=True,
                             dtype=_dtype_code(Q), softmax_scale=softmax_scale, max_seqlen=max_seqlen)
        dev = Q.device
        z = torch.empty((H_q, T), dtype=torch.float32, device=dev)
        expiry = torch.empty((H_q, T), dtype=torch.int32, device=dev)
        mask = torch.empty(B.dma_mask_bytes(shape), dtype=torch.uint8, device=dev)
        ws_bytes = B.dma_workspace_bytes(shape)
        ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)
        O = torch.empty_like(Q)
        LSE = torch.empty((H_q, T), dtype=torch.float32, device=dev)
        xhead = K.shape[1] > 1 and W.shape[1] == K.shape[1] * d
        if xhead:
            B.dma_scores_xhead(shape, V, W, A, z)
        Wm, Am = (None, None) if xhead else (W, A)          # cross-head: the scores are supplied to dma_mask_gen
        if bias is None:
            B.dma_mask_gen(shape, V, Wm, Am, cu_seqlens, z, expiry, None, mask)
        else:
            B.dma_mask_gen_bias(shape, V, Wm, Am, cu_seqlens, bias, bias_heads, bias_per_token, z, expiry, None, mask)
        B.dma_fwd(shape, Q, K, V, z, expiry, mask, cu_seqlens, O, LSE, ws, ws_bytes)
        ctx.save_for_backward(Q, K, V, W, A, cu_seqlens, z, expiry, mask, O, LSE)
        ctx.shape, ctx.ws, ctx.ws_bytes, ctx.xhead = shape, ws, ws_bytes, xhead
        ctx.bias_form = None if bias is None else (bias_heads, bias_per_token, tuple(bias.shape))
        return O

    @staticmethod
    def backward(ctx, dO):
        Q, K, V, W, A, cu_seqlens, z, expiry, mask, O, LSE = ctx.saved_tensors
        shape = ctx.shape
        dO = dO.contiguous()
        dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
        dz = torch.empty_like(z)
        dW, dA = torch.empty_like(W), torch.empty_like(A)
        B.dma_bwd(shape, Q, K, V, O, dO, LSE, z, expiry, mask, cu_seqlens, dQ, dK, dV, dz, ctx.ws, ctx.ws_bytes)
        # dz -> dW, dA, and the part of dV that flows through the content scores, added in place
        (B.dma_scores_xhead_bwd if ctx.xhead else B.dma_mask_bwd)(shape, V, W, A, dz, dW, dA, dV, True)
        dbias = None
        if ctx.bias_form is not None:   # the bias enters the score like z: its gradient is dz, reduced over what shares it
            bias_heads, bias_per_token, bshape = ctx.bias_form
            dbias = torch.empty(bshape, dtype=torch.float32, device=dz.device)
            B.dma_bias_bwd(shape, dz, cu_seqlens, bias_heads, bias_per_token, dbias)
        return dQ, dK, dV, dW, dA, None, None, None, None, dbias


def dynamic_mask_attention(Q, K, V, W, A, cu_seqlens, k, max_seqlen=0, softmax_scale=0.0, bias=None):
    """Functional form; see DynamicMaskAttentionFunction.  bias (optional, differentiable): a further
    additive attention bias per key, [H_q or 1, T] or [H_q or 1, max_seqlen] (Section 1: biases with
    batch, head and query broadcasting); it does not take part in the selection of the kept keys."""
    return DynamicMaskAttentionFunction.apply(Q, K, V, W, A, cu_seqlens, k, max_seqlen, softmax_scale, bias)


class DynamicMaskAttention(torch.nn.Module):
    """The attention core of a DMA layer (the part between the QKV projections and the output
    projection).  Parameters: the score projection `W` [H_q, d] (the paper's Delta taken per head;
    [H_q, H_kv * d], the full tensor, with cross_head=True) and the gate `A` [H_q].  Their
    initialisation is a choice of this module, not the paper's: W ~ N(0, 1 / fan-in), A = -1, which
    keeps the initial scores in (0, 1) and close together.

    forward(q, k, v): [B, L, H, d] batches (each sequence its own document), or packed [T, H, d]
    tensors with cu_seqlens.
    """

    def __init__(self, num_heads, num_kv_heads, head_dim, keep_window, softmax_scale=None, device=None,
                 cross_head=False):
        super().__init__()
        if num_heads % num_kv_heads:
            raise ValueError("num_heads must be a multiple of num_kv_heads")
        self.num_heads, self.num_kv_heads, self.head_dim = num_heads, num_kv_heads, head_dim
        self.keep_window = int(keep_window)
        self.softmax_scale = 0.0 if softmax_scale is None else float(softmax_scale)
        fan_in = head_dim * (num_kv_heads if cross_head else 1)   # cross_head: the full Delta of Eq. 3
        self.W = torch.nn.Parameter(torch.randn(num_heads, fan_in, dtype=torch.float32, device=device)
                                    / math.sqrt(fan_in))
        self.A = torch.nn.Parameter(torch.full((num_heads,), -1.0, dtype=torch.float32, device=device))

    def forward(self, q, k, v, cu_seqlens=None, max_seqlen=0):
        if q.dim() == 4:
            if cu_seqlens is not None:
                raise ValueError("cu_seqlens goes with packed [T, H, d] inputs")
            Bsz, L = q.shape[0], q.shape[1]
            cu = torch.arange(0, (Bsz + 1) * L, L, dtype=torch.int32, device=q.device)
            o = dynamic_mask_attention(q.reshape(Bsz * L, *q.shape[2:]), k.reshape(Bsz * L, *k.shape[2:]),
                                       v.reshape(Bsz * L, *v.shape[2:]), self.W, self.A, cu,
                                       self.keep_window, L, self.softmax_scale)
            return o.view(Bsz, L, *q.shape[2:])
        if cu_seqlens is None:
            raise ValueError("packed inputs need cu_seqlens")
        return dynamic_mask_attention(q, k, v, self.W, self.A, cu_seqlens, self.keep_window, max_seqlen,
                                      self.softmax_scale)
