"""torch.autograd face of the attention kernels: `attention(q, k, v, ...)` runs ie_attn_fwd and, in
backward, ie_attn_bwd on the saved o and log-sum-exp (the probabilities are recomputed, Sec. 3.1).
Only tensor bookkeeping happens here; there is no fallback path."""
import torch

from . import binding


class _Attention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, k, v, scale, causal, cu_seqlens):
        q, k, v = q.contiguous(), k.contiguous(), v.contiguous()
        o, lse = binding.attn_fwd(q, k, v, scale, causal, cu_seqlens)
        ctx.save_for_backward(q, k, v, o, lse)
        ctx.cu_seqlens, ctx.scale, ctx.causal = cu_seqlens, scale, causal
        ctx.mark_non_differentiable(lse)
        return o, lse

    @staticmethod
    def backward(ctx, dout, _dlse):
        q, k, v, o, lse = ctx.saved_tensors
        dq, dk, dv = binding.attn_bwd(q, k, v, o, dout.contiguous(), lse, ctx.scale, ctx.causal, ctx.cu_seqlens)
        return dq, dk, dv, None, None, None


def attention(q, k, v, scale=None, causal=True, cu_seqlens=None, return_lse=False):
    """Exact softmax attention of q [B,S,Hq,D] against k, v [B,S,Hkv,D] (bf16, on the GPU), differentiable
    in q, k and v.  `cu_seqlens` (int32, on the GPU) packs several documents into one sequence (B = 1)."""
    if scale is None:
        scale = q.shape[-1] ** -0.5
    o, lse = _Attention.apply(q, k, v, float(scale), bool(causal), cu_seqlens)
    return (o, lse) if return_lse else o
