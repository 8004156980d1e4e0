"""Jagged flash attention as differentiable torch functions of q, k and v (paper Section 2.2: the operators have a
forward and a backward so that they can be trained through).

Argument marshalling only: the forward of each function is the library's forward entry point, its backward the
library's backward entry point on the tensors the forward saved; nothing is computed here, and a missing library
raises as everywhere in the binding.

    out = jagged_flash_attention(q, k, v, offsets, max_len)                      # self attention, causal=True for the causal variant
    out = jagged_flash_cross_attention(q, k, v, offsets_q, offsets_kv, max_len_q, max_len_kv)

q, k, v: [rows, H, D] bf16 or fp32 on the GPU, contiguous; offsets: int64 [B + 1] on the GPU.  Gradients flow to q, k
and v; offsets and the length bounds are not differentiable.
"""
import torch

from . import binding

__all__ = ["jagged_flash_attention", "jagged_flash_cross_attention"]


class _SelfAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, k, v, offsets, max_len, causal):
        out, lse = binding.jfa_forward(q, k, v, offsets, max_len, causal=causal)
        ctx.save_for_backward(q, k, v, out, lse, offsets)
        ctx.max_len, ctx.causal = max_len, causal
        return out

    @staticmethod
    def backward(ctx, dout):
        q, k, v, out, lse, offsets = ctx.saved_tensors
        dq, dk, dv, _ = binding.jfa_backward(q, k, v, out, dout.contiguous(), lse, offsets, ctx.max_len, causal=ctx.causal)
        return dq, dk, dv, None, None, None


class _CrossAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, k, v, offsets_q, offsets_kv, max_len_q, max_len_kv):
        out, lse = binding.jfa_forward_cross(q, k, v, offsets_q, offsets_kv, max_len_q, max_len_kv)
        ctx.save_for_backward(q, k, v, out, lse, offsets_q, offsets_kv)
        ctx.max_len_q, ctx.max_len_kv = max_len_q, max_len_kv
        return out

    @staticmethod
    def backward(ctx, dout):
        q, k, v, out, lse, offsets_q, offsets_kv = ctx.saved_tensors
        dq, dk, dv, _ = binding.jfa_backward_cross(q, k, v, out, dout.contiguous(), lse, offsets_q, offsets_kv,
                                                   ctx.max_len_q, ctx.max_len_kv)
        return dq, dk, dv, None, None, None, None


def jagged_flash_attention(q, k, v, offsets, max_len: int, causal: bool = False):
    """softmax(Q K^T / sqrt(D)) V per sample and head over the jagged rows that `offsets` delimits (Section 2.1)."""
    return _SelfAttention.apply(q, k, v, offsets, int(max_len), bool(causal))


def jagged_flash_cross_attention(q, k, v, offsets_q, offsets_kv, max_len_q: int, max_len_kv: int):
    """The queries of sample b (rows of offsets_q) attend to its keys and values (rows of offsets_kv)."""
    return _CrossAttention.apply(q, k, v, offsets_q, offsets_kv, int(max_len_q), int(max_len_kv))
