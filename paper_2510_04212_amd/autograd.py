"""torch.autograd wrapper over the C ABI: `attention(q, k, v, ...)` is differentiable.

Argument marshalling only: the forward pass is attn_fwd / attn_fwd_strided and the backward
pass attn_bwd / attn_bwd_strided of the library (Alg. 1 or Alg. 3 forward, Alg. 2 backward of
arXiv 2510.04212); nothing is computed here.  q, k, v are bfloat16 CUDA tensors of logical
shape [B, H, N, d]; they may be contiguous or share any batch / head / row strides with a
contiguous last dimension (for instance `x.view(B, N, H, d).permute(0, 2, 1, 3)`), in which case
no copy is made.  k and v may have fewer heads than q (grouped-query attention), or a different
sequence length (the causal mask is then aligned at the bottom right).
"""
import math

import torch

from . import binding


def _same_layout(*ts):
    s0 = ts[0].stride()
    return all(t.stride() == s0 and t.shape == ts[0].shape for t in ts)


class _FlashAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, k, v, causal, softmax_scale, variant, beta, eps):
        if k.shape[1] != q.shape[1]:        # grouped-query attention: fewer key/value heads
            q, k, v = q.contiguous(), k.contiguous(), v.contiguous()
            o, lse = binding.attn_fwd_gqa(q, k, v, causal, softmax_scale, variant, beta, eps)
            ctx.save_for_backward(q, k, v, o, lse)
            ctx.args = (causal, softmax_scale, variant, "gqa")
            return o
        if k.shape[2] != q.shape[2]:        # different numbers of queries and keys
            q, k, v = q.contiguous(), k.contiguous(), v.contiguous()
            o, lse = binding.attn_fwd_rect(q, k, v, causal, softmax_scale, variant, beta, eps)
            ctx.save_for_backward(q, k, v, o, lse)
            ctx.args = (causal, softmax_scale, variant, "rect")
            return o
        strided = not (q.is_contiguous() and k.is_contiguous() and v.is_contiguous())
        if strided and not (_same_layout(q, k, v) and q.stride(3) == 1):
            q, k, v = q.contiguous(), k.contiguous(), v.contiguous()
            strided = False
        if strided:
            o, lse = binding.attn_fwd_strided(q, k, v, causal, softmax_scale, variant, beta, eps)
        else:
            o, lse = binding.attn_fwd(q, k, v, causal, softmax_scale, variant, beta, eps)
        ctx.save_for_backward(q, k, v, o, lse)
        ctx.args = (causal, softmax_scale, variant, strided)
        return o

    @staticmethod
    def backward(ctx, do):
        q, k, v, o, lse = ctx.saved_tensors
        causal, softmax_scale, variant, strided = ctx.args
        if strided == "gqa":
            dq, dk, dv = binding.attn_bwd_gqa(q, k, v, o, do.contiguous(), lse, causal, softmax_scale, variant)
        elif strided == "rect":
            dq, dk, dv = binding.attn_bwd_rect(q, k, v, o, do.contiguous(), lse, causal, softmax_scale, variant)
        elif strided:
            if do.stride() != q.stride():
                d2 = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
                d2.copy_(do)
                do = d2
            dq, dk, dv = binding.attn_bwd_strided(q, k, v, o, do, lse, causal, softmax_scale, variant)
        else:
            dq, dk, dv = binding.attn_bwd(q, k, v, o, do.contiguous(), lse, causal, softmax_scale, variant)
        return dq, dk, dv, None, None, None, None, None


def attention(q, k, v, causal=True, softmax_scale=None, variant=binding.MITIGATED, beta=None, eps=None):
    """softmax(softmax_scale * q k^T) v with gradients, on the HIP kernels.

    variant: binding.STANDARD (Alg. 1), binding.MITIGATED (Alg. 3, the default: the paper's
    fix for the rounding bias) or binding.MITIGATED_ROW (its rule on the whole row).
    softmax_scale defaults to 1/sqrt(d)."""
    if softmax_scale is None:
        softmax_scale = 1.0 / math.sqrt(q.shape[-1])
    return _FlashAttention.apply(q, k, v, bool(causal), float(softmax_scale), int(variant), beta, eps)
