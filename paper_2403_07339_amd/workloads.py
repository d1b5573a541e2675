"""Seeded synthetic GEMM operands shaped like the paper's Transformer workloads.

This module only *draws inputs*: it contains none of the method's arithmetic
(no rounding to integers, no unpacking, no products) and imports neither the HIP
binding nor the CPU checker, so both can be fed from it.

The paper (arXiv 2403.07339, Sec. 4.2 and its unpack-ratio tables) measures on
real LLaMA-7B / ViT / RoBERTa activations, weights and gradients, which are not
available here.  The five workloads below stand in for them: same GEMM shapes,
fp32 values, and heavy hitters concentrated in a few channels or scattered as a
tiny fraction of the entries, which is the structure the paper reports
(Sec. 3 and the Summary of Sec. 4).

Orientation (Sec. 1, Eq. gemm): A is n x d, B is h x d, C = A B^T; the second
index is the contracted one.  A Linear layer Y = X W^T has A = X, B = W stored
[out, in].

Draw order per workload, all from one ``torch.Generator`` seeded with
``index - 1``: A values, A heavy-hitter positions, B values, B heavy-hitter
positions.  The per-tensor step is ``scale = float32(4 * std / 127)`` with the
population standard deviation taken in float64 over the whole tensor.
"""
from __future__ import annotations

from dataclasses import dataclass

import torch

ROW, COL, BOTH = 0, 1, 2
STRATEGY_NAMES = {ROW: "row", COL: "col", BOTH: "both"}


@dataclass
class Workload:
    name: str
    A: torch.Tensor          # fp32, logical shape (n, d); may be a strided (transposed) view
    B: torch.Tensor          # fp32, logical shape (h, d); may be a strided view
    scale_a: float           # exactly representable in float32
    scale_b: float
    b: int
    strategy_a: int
    strategy_b: int

    @property
    def n(self) -> int:
        return self.A.shape[0]

    @property
    def d(self) -> int:
        return self.A.shape[1]

    @property
    def h(self) -> int:
        return self.B.shape[0]

    @property
    def ops(self) -> int:
        """2 n d h of the original GEMM."""
        return 2 * self.n * self.d * self.h


def rtn_scale(x: torch.Tensor) -> float:
    """float32(4 * std / 127), std = population standard deviation in float64."""
    std = x.double().std(unbiased=False).item()
    return float(torch.tensor(4.0 * std / 127.0, dtype=torch.float64).to(torch.float32).item())


def _normal(g, rows, cols, std=1.0):
    x = torch.randn(rows, cols, generator=g, dtype=torch.float32)
    if std != 1.0:
        x.mul_(std)
    return x


def _scale_columns(x, g, count, factor):
    idx = torch.randperm(x.shape[1], generator=g)[:count]
    x[:, idx] *= factor
    return idx


def _scale_positions(x, g, fraction, factor):
    total = x.numel()
    count = int(round(fraction * total))
    idx = torch.randperm(total, generator=g)[:count]
    flat = x.view(-1)
    flat[idx] *= factor
    return idx


def _student_t3(g, rows, cols):
    z = torch.randn(rows, cols, generator=g, dtype=torch.float32)
    chi2 = torch.zeros(rows, cols, dtype=torch.float32)
    for _ in range(3):
        chi2 += torch.randn(rows, cols, generator=g, dtype=torch.float32) ** 2
    return z / torch.sqrt(chi2 / 3.0)


WORKLOAD_NAMES = {
    1: "tiny-256x256x256-b8-both/both",
    2: "vit-b-fc1-12608x768x3072-b8-row/col",
    3: "llama7b-up-4096x4096x11008-b8-both/both",
    4: "wgrad-4096x8192x4096-b8-both/both",
    5: "lowbit-4096x4096x4096-b4-row/col",
}


def make(index: int) -> Workload:
    """The index-th (1-based) benchmark workload."""
    g = torch.Generator(device="cpu")
    g.manual_seed(index - 1)
    if index == 1:
        A = _normal(g, 256, 256)
        _scale_positions(A, g, 0.005, 64.0)
        B = _normal(g, 256, 256)
        _scale_positions(B, g, 0.005, 64.0)
        b, sa, sb = 8, BOTH, BOTH
    elif index == 2:
        A = _normal(g, 12608, 768)
        _scale_columns(A, g, 6, 40.0)
        B = _normal(g, 3072, 768, 0.02)
        b, sa, sb = 8, ROW, COL
    elif index == 3:
        A = _normal(g, 4096, 4096)
        _scale_columns(A, g, round(0.005 * 4096), 100.0)
        B = _normal(g, 11008, 4096, 0.02)
        _scale_positions(B, g, 0.001, 20.0)
        b, sa, sb = 8, BOTH, BOTH
    elif index == 4:
        dY = _student_t3(g, 8192, 4096)          # stored [tokens, out]
        X = _normal(g, 8192, 4096)               # stored [tokens, in]
        _scale_columns(X, g, round(0.005 * 4096), 50.0)
        A, B = dY.t(), X.t()                     # dW = dY^T X: contraction over tokens, strided views
        b, sa, sb = 8, BOTH, BOTH
    elif index == 5:
        A = _normal(g, 4096, 4096)
        _scale_columns(A, g, 6, 40.0)
        B = _normal(g, 4096, 4096, 0.02)
        b, sa, sb = 4, ROW, COL
    else:
        raise ValueError(f"no workload {index}")
    return Workload(WORKLOAD_NAMES[index], A, B, rtn_scale(A), rtn_scale(B), b, sa, sb)


def small(seed: int, n: int, d: int, h: int, kind: str = "scattered", b: int = 8,
          strategy_a: int = BOTH, strategy_b: int = BOTH) -> Workload:
    """Small fp32 operands with the same heavy-hitter structures, for element-by-element parity.

    kind: "scattered" (a small fraction of positions scaled up), "channels" (a few contracted
    columns scaled up), "rows" (a few rows scaled up), "heavy" (Student-t, nu = 3), "clean" (none),
    "deep" (scattered entries large enough to need three or more digits).
    """
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)

    def one(rows, cols):
        x = _normal(g, rows, cols)
        if kind == "scattered":
            _scale_positions(x, g, 0.01, 64.0)
        elif kind == "channels":
            _scale_columns(x, g, max(1, cols // 64), 50.0)
        elif kind == "rows":
            idx = torch.randperm(rows, generator=g)[:max(1, rows // 64)]
            x[idx, :] *= 50.0
        elif kind == "heavy":
            x = _student_t3(g, rows, cols)
        elif kind == "deep":
            _scale_positions(x, g, 0.01, 64.0)
            _scale_positions(x, g, 0.002, 4096.0)
        elif kind != "clean":
            raise ValueError(kind)
        return x

    A = one(n, d)
    B = one(h, d)
    return Workload(f"small-{kind}-{n}x{d}x{h}-b{b}", A, B, rtn_scale(A), rtn_scale(B), b,
                    strategy_a, strategy_b)
