"""A linear layer whose three GEMMs run on the exact low-bit integer path.

Sec. 1 ("Notations") of arXiv 2403.07339 lists the GEMMs of a Transformer; for a linear layer they are

    Y      = X  W^T          (forward)
    grad_X = grad_Y  W       (backward, input)
    grad_W = grad_Y^T  X     (backward, weight)

Each is computed as in Sec. 2: both operands are RTN-quantised with the step alpha_p / (0.5 beta)
(Eq. (quantized_A)), the integer GEMM is evaluated exactly with b-bit digits (Sec. 4: plan, unpack,
int8 MFMA GEMM, recombination) and the result is scaled back (Eq. (quantized_gemm)) -- all inside
``imunpack_gemm_batched`` of the C ABI, which keeps the steps on the device.  The weights stay in fp32
(master copy).  Integration only: every arithmetic step of the method runs in the HIP library.
"""
from __future__ import annotations

from dataclasses import dataclass

import torch

from . import binding as imu


@dataclass
class QuantConfig:
    """beta_*: number of integers that cover [-alpha_p, alpha_p] (Eq. (quantized_A)) for activations,
    weights and gradients; p: the percentile; b: bit width of the unpacked integers (Sec. 4);
    strategies: how the first / second operand of each GEMM is unpacked."""
    beta_x: float = 255.0
    beta_w: float = 255.0
    beta_g: float = 1023.0
    p: float = 95.0
    b: int = 8
    strategy_a: int = imu.BOTH
    strategy_b: int = imu.BOTH


def quantized_matmul(A: torch.Tensor, B: torch.Tensor, beta_a: float, beta_b: float, cfg: QuantConfig) -> torch.Tensor:
    """A B^T for A: n x d, B: h x d (fp32 device tensors, any strides), on the exact integer path: one
    call of the library's batched entry point with a batch of one.  The RTN steps alpha_p / (0.5 beta) are
    formed and used on the device; nothing of the method is computed here."""
    return imu.imunpack_gemm_batched(A, B, cfg.p, beta_a, beta_b, cfg.b, cfg.strategy_a, cfg.strategy_b)


class _LinearFunction(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, weight, bias, cfg):
        x2 = x.reshape(-1, x.shape[-1])
        y = quantized_matmul(x2, weight, cfg.beta_x, cfg.beta_w, cfg)
        if bias is not None:
            y = y + bias
        ctx.save_for_backward(x2, weight)
        ctx.cfg = cfg
        ctx.has_bias = bias is not None
        ctx.x_shape = x.shape
        return y.reshape(*x.shape[:-1], weight.shape[0])

    @staticmethod
    def backward(ctx, gy):
        x2, weight = ctx.saved_tensors
        cfg = ctx.cfg
        g2 = gy.reshape(-1, gy.shape[-1]).contiguous()
        gx = gw = gb = None
        if ctx.needs_input_grad[0]:   # grad_X = grad_Y W: the contraction runs over the output features
            gx = quantized_matmul(g2, weight.t(), cfg.beta_g, cfg.beta_w, cfg).reshape(ctx.x_shape)
        if ctx.needs_input_grad[1]:   # grad_W = grad_Y^T X: the contraction runs over the tokens
            gw = quantized_matmul(g2.t(), x2.t(), cfg.beta_g, cfg.beta_x, cfg)
        if ctx.has_bias and ctx.needs_input_grad[2]:
            gb = g2.sum(0)
        return gx, gw, gb, None


class IMUnpackLinear(torch.nn.Module):
    """``torch.nn.Linear`` with the three GEMMs on the exact low-bit integer path (fp32 parameters)."""

    def __init__(self, in_features: int, out_features: int, bias: bool = True, cfg: QuantConfig | None = None,
                 device=None):
        super().__init__()
        ref = torch.nn.Linear(in_features, out_features, bias=bias, device=device, dtype=torch.float32)
        self.weight = ref.weight
        self.bias = ref.bias
        self.cfg = cfg or QuantConfig()

    def forward(self, x: torch.Tensor) -> torch.Tensor:
        return _LinearFunction.apply(x, self.weight, self.bias, self.cfg)
