"""torch.autograd wrappers around the C-ABI calls (argument marshalling only).

``window_attention(q, k, v, heads, scale, bias, mask)`` takes [N, L, C] tensors;
``window_attention_qkv(qkv, scale, bias, mask)`` takes the fused projection output
[N, L, 3, heads, d] and reads q, k, v in place through row strides (no permute, no copy);
its backward writes dq, dk, dv straight into one [N, L, 3, heads, d] gradient tensor.
The backward kernels need nothing from the forward but its inputs (paper Algorithm 2).
Both take the mask either as a dense fp32 ``mask`` [nW, L, L] or as int32 region ``labels``
[nW, L] with a ``mask_value`` (the kernels then form the mask themselves).
"""
from __future__ import annotations

import torch

from . import binding


def _check_dbias_supported(q, heads, bias):
    if bias is not None and bias.requires_grad:
        N, L, C = q.shape
        if binding.fwa_backward_workspace_bytes(max(N, 1), L, C, heads, binding._dtype_code(q), True) == 0 and N > 0:
            raise NotImplementedError("the gradient of the bias is not available for this shape and dtype")


class _WindowAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, k, v, bias, mask, heads, scale, labels, mask_value):
        ctx.save_for_backward(q, k, v, bias, mask, labels)
        ctx.heads, ctx.scale, ctx.mask_value = heads, scale, mask_value
        return binding.fwa_forward(q, k, v, heads, scale, bias, mask, labels=labels, mask_value=mask_value)

    @staticmethod
    def backward(ctx, d_o):
        q, k, v, bias, mask, labels = ctx.saved_tensors
        want_db = bias is not None and ctx.needs_input_grad[3]
        if not d_o.is_contiguous():
            d_o = d_o.contiguous()
        dq, dk, dv, db = binding.fwa_backward(q, k, v, d_o, ctx.heads, ctx.scale, bias, mask, want_dbias=want_db,
                                              labels=labels, mask_value=ctx.mask_value)
        return dq, dk, dv, db, None, None, None, None, None


class _WindowAttentionQKV(torch.autograd.Function):
    @staticmethod
    def forward(ctx, qkv, bias, mask, scale, labels, mask_value):
        N, L, three, heads, d = qkv.shape
        ctx.save_for_backward(qkv, bias, mask, labels)
        ctx.scale, ctx.mask_value = scale, mask_value
        q, k, v = (qkv[:, :, t].reshape(N, L, heads * d) for t in range(3))  # views: row stride 3 C
        return binding.fwa_forward(q, k, v, heads, scale, bias, mask, labels=labels, mask_value=mask_value)

    @staticmethod
    def backward(ctx, d_o):
        qkv, bias, mask, labels = ctx.saved_tensors
        N, L, three, heads, d = qkv.shape
        want_db = bias is not None and ctx.needs_input_grad[1]
        if not d_o.is_contiguous():
            d_o = d_o.contiguous()
        q, k, v = (qkv[:, :, t].reshape(N, L, heads * d) for t in range(3))
        dqkv = torch.empty_like(qkv)
        out = tuple(dqkv[:, :, t].reshape(N, L, heads * d) for t in range(3))
        _, _, _, db = binding.fwa_backward(q, k, v, d_o, heads, ctx.scale, bias, mask, want_dbias=want_db, out=out,
                                           labels=labels, mask_value=ctx.mask_value)
        return dqkv, db, None, None, None, None


def window_attention(q, k, v, heads: int, scale: float, bias=None, mask=None, labels=None, mask_value: float = -100.0):
    """softmax(scale * Q K^T + bias + mask) V per window and head, differentiable in q, k, v and bias."""
    _check_dbias_supported(q, heads, bias)
    return _WindowAttention.apply(q, k, v, bias, mask, heads, scale, labels, float(mask_value))


def window_attention_qkv(qkv, scale: float, bias=None, mask=None, labels=None, mask_value: float = -100.0):
    """The same on a fused, contiguous [N, L, 3, heads, d] tensor; returns [N, L, heads * d]."""
    if qkv.dim() != 5 or qkv.shape[2] != 3 or not qkv.is_contiguous():
        raise ValueError("qkv must be a contiguous [N, L, 3, heads, d] tensor")
    N, L, _, heads, d = qkv.shape
    _check_dbias_supported(qkv[:, :, 0].reshape(N, L, heads * d), heads, bias)
    return _WindowAttentionQKV.apply(qkv, bias, mask, scale, labels, float(mask_value))
