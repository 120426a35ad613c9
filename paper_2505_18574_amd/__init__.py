"""MI355X (gfx950) implementation of the dense tensor operations that arxiv
2505.18574 optimises: int8 GEMM and convolution with the int8 accelerator's
bias / scale-down / saturate / ReLU output stage, bf16 GEMM, and batched small
fp32 linear algebra.

``paper_2505_18574_amd.ops`` is the thin binding over the C-ABI library built
from ``csrc/``; ``paper_2505_18574_amd.inputs`` holds the seeded workload
generators.  Importing the package loads nothing; the first use of ``ops``
loads the HIP library and raises if it has not been built.
"""

__all__ = ["inputs", "ops"]
