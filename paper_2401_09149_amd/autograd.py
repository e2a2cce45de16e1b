"""torch.autograd face of the kernels: `attention(q, k, v, ...)` runs ie_attn_fwd and, in backward, ie_attn_bwd
on the saved o and log-sum-exp (the probabilities are recomputed, Sec. 3.2); `linear(x, w)` runs the three
products of a Linear module without bias (Sec. 4.2).  Only tensor bookkeeping happens here; there is no
fallback path."""
import torch

from . import binding


class _Attention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, k, v, scale, causal, cu_seqlens, workspace, recompute, stored_ds):
        q, k, v = q.contiguous(), k.contiguous(), v.contiguous()
        o, lse = binding.attn_fwd(q, k, v, scale, causal, cu_seqlens)
        if recompute:   # keep the inputs only; the outputs handed to the caller are not referenced from here
            ctx.save_for_backward(q, k, v)
        else:
            ctx.save_for_backward(q, k, v, o, lse)
        ctx.cu_seqlens, ctx.scale, ctx.causal, ctx.workspace, ctx.stored_ds = cu_seqlens, scale, causal, workspace, stored_ds
        ctx.mark_non_differentiable(lse)
        return o, lse

    @staticmethod
    def backward(ctx, dout, _dlse):
        if len(ctx.saved_tensors) == 3:   # activation recomputation: an additional forward pass (Sec. 2.3)
            q, k, v = ctx.saved_tensors
            o, lse = binding.attn_fwd(q, k, v, ctx.scale, ctx.causal, ctx.cu_seqlens)
        else:
            q, k, v, o, lse = ctx.saved_tensors
        dq, dk, dv = binding.attn_bwd(q, k, v, o, dout.contiguous(), lse, ctx.scale, ctx.causal, ctx.cu_seqlens,
                                      workspace=ctx.workspace, stored_ds=ctx.stored_ds)
        return dq, dk, dv, None, None, None, None, None, None


def attention(q, k, v, scale=None, causal=True, cu_seqlens=None, return_lse=False, workspace=None, recompute=False,
              stored_ds=False):
    """Exact softmax attention of q [B,S,Hq,D] against k, v [B,S,Hkv,D] (bf16, on the GPU), differentiable
    in q, k and v.  `cu_seqlens` (int32, on the GPU) packs several documents into one sequence (B = 1).
    `workspace`: a uint8 GPU tensor for the backward pass, typically one binding.alloc_bwd_workspace(q, k)
    shared by all layers; by default one is allocated per call.  `stored_ds`: take the backward path that keeps dS
    in the workspace (binding.alloc_bwd_workspace(q, k, fast=True): B*Hq*S*(S+128) bytes more).  `recompute`: activation recomputation for this module (Sec. 2.3) — o and the log-sum-exp
    are not kept for the backward pass, which runs the forward kernel once more instead (bit-identical values)."""
    if scale is None:
        scale = q.shape[-1] ** -0.5
    o, lse = _Attention.apply(q, k, v, float(scale), bool(causal), cu_seqlens, workspace, bool(recompute), bool(stored_ds))
    return (o, lse) if return_lse else o


class _Linear(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, w):
        lead = x.shape[:-1]
        x2 = x.reshape(-1, x.shape[-1]).contiguous()
        w = w.contiguous()
        y = torch.empty((x2.shape[0], w.shape[0]), dtype=torch.bfloat16, device=x.device)
        binding.ie_linear_fwd(x2, w, y)
        ctx.save_for_backward(x2, w)
        ctx.lead = lead
        return y.reshape(*lead, w.shape[0])

    @staticmethod
    def backward(ctx, dy):
        x2, w = ctx.saved_tensors
        dy2 = dy.reshape(-1, dy.shape[-1]).contiguous()
        dx = dw = None
        if ctx.needs_input_grad[0]:
            dx = torch.empty_like(x2)
            binding.ie_linear_bwd_input(dy2, w, dx)
            dx = dx.reshape(*ctx.lead, x2.shape[1])
        if ctx.needs_input_grad[1]:
            dw = torch.empty_like(w)
            binding.ie_linear_bwd_weight(dy2, x2, dw)
        return dx, dw


def linear(x, w):
    """y = x w^T for x [..., K] and w [N, K] (bf16, on the GPU), differentiable in both.  The token count (product of
    the leading dimensions) must be a multiple of 64 for the weight gradient, K and N multiples of 64."""
    return _Linear.apply(x, w)
