"""MI355X-native exact low-bit integer GEMM (IM-Unpack, arXiv 2403.07339).

``paper_2403_07339_amd.binding`` wraps the C-ABI HIP library (it raises if the
library has not been built); ``paper_2403_07339_amd.workloads`` draws the seeded
synthetic operands; ``paper_2403_07339_amd.linear`` is a linear layer and
``paper_2403_07339_amd.attention`` self-attention (autograd functions and modules) whose GEMMs run
through the binding.  Nothing is imported eagerly so that the input generators can
be used on machines without the built library.
"""
__all__ = ["binding", "workloads", "linear", "attention"]
