"""Self-attention whose six GEMMs run on the exact low-bit integer path.

Sec. 1 ("Notations") of arXiv 2403.07339 lists, beside the GEMMs of the linear layer, those of self-attention,

    P = Q K^T            O = M V                 (forward;  M = softmax(P), scaling factors omitted there)
    grad_Q = grad_P K    grad_K = grad_P^T Q     grad_M = grad_O V^T    grad_V = M^T grad_O   (backward)

one set per sequence and head.  Each is computed as in Sec. 2 and Sec. 4 by ``imunpack_gemm_batched``:
both operands RTN-quantised with their own step alpha_p / (0.5 beta), the integer GEMM evaluated exactly
with b-bit digits, the result scaled back.  Every matrix of every sequence and head is an operand of its
own (its own percentile, its own plan); the operands are strided views, nothing is copied or transposed
on the way in.  The softmax and its derivative are not GEMMs and stay in fp32 torch arithmetic.
Integration on top of the C ABI binding: one strided-batched call per GEMM of the layer.
"""
from __future__ import annotations

import math

import torch

from . import binding as imu
from .linear import QuantConfig


def quantized_bmm(A: torch.Tensor, B: torch.Tensor, beta_a: float, beta_b: float, cfg: QuantConfig) -> torch.Tensor:
    """A B^T over the leading dimensions: A [..., n, d], B [..., h, d] (fp32 device tensors, any strides,
    equal leading shapes) -> [..., n, h]; every matrix pair is one exact integer GEMM.  One call of the
    library's strided-batched entry point for all sequences and heads."""
    if A.shape[:-2] != B.shape[:-2] or A.shape[-1] != B.shape[-1]:
        raise ValueError(f"shapes {tuple(A.shape)} and {tuple(B.shape)} do not form a batched A B^T")
    return imu.imunpack_gemm_batched(A, B, cfg.p, beta_a, beta_b, cfg.b, cfg.strategy_a, cfg.strategy_b)


class _AttentionFunction(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, k, v, scale, cfg, trace):
        p = quantized_bmm(q, k, cfg.beta_x, cfg.beta_x, cfg)                     # P = Q K^T
        m = torch.softmax(p * scale, dim=-1)
        o = quantized_bmm(m, v.transpose(-1, -2), cfg.beta_x, cfg.beta_x, cfg)   # O = M V
        ctx.save_for_backward(q, k, v, m)
        ctx.scale, ctx.cfg, ctx.trace = scale, cfg, trace
        if trace is not None:
            trace.update(P=p, M=m, O=o)
        return o

    @staticmethod
    def backward(ctx, go):
        q, k, v, m = ctx.saved_tensors
        cfg, trace = ctx.cfg, ctx.trace
        go = go.contiguous()
        gq = gk = gv = None
        if ctx.needs_input_grad[2]:   # grad_V = M^T grad_O: the contraction runs over the queries
            gv = quantized_bmm(m.transpose(-1, -2), go.transpose(-1, -2), cfg.beta_x, cfg.beta_g, cfg)
        if ctx.needs_input_grad[0] or ctx.needs_input_grad[1]:
            gm = quantized_bmm(go, v, cfg.beta_g, cfg.beta_x, cfg)                # grad_M = grad_O V^T
            gp = (gm - (gm * m).sum(-1, keepdim=True)) * m * ctx.scale             # softmax and the scaling of P
            if trace is not None:
                trace.update(grad_M=gm, grad_P=gp)
            if ctx.needs_input_grad[0]:   # grad_Q = grad_P K: the contraction runs over the keys
                gq = quantized_bmm(gp, k.transpose(-1, -2), cfg.beta_g, cfg.beta_x, cfg)
            if ctx.needs_input_grad[1]:   # grad_K = grad_P^T Q: the contraction runs over the queries
                gk = quantized_bmm(gp.transpose(-1, -2), q.transpose(-1, -2), cfg.beta_g, cfg.beta_x, cfg)
        return gq, gk, gv, None, None, None


class IMUnpackAttention(torch.nn.Module):
    """softmax(Q K^T / sqrt(d_head)) V for q, k, v of shape [..., tokens, d_head] (any leading dimensions:
    sequences, heads), all six GEMMs of forward and backward on the exact low-bit integer path.  The
    projections around it are linear layers (``linear.IMUnpackLinear``).  ``trace``: a dict that, if given,
    receives the intermediate matrices P, M, O, grad_M, grad_P of the last call (for inspection)."""

    def __init__(self, cfg: QuantConfig | None = None, trace: dict | None = None):
        super().__init__()
        self.cfg = cfg or QuantConfig()
        self.trace = trace

    def forward(self, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor) -> torch.Tensor:
        return _AttentionFunction.apply(q, k, v, 1.0 / math.sqrt(q.shape[-1]), self.cfg, self.trace)
