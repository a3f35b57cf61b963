"""CPU oracle for the FP8 Smooth-SwiGLU MLP block.  TEST INFRASTRUCTURE ONLY.

A plain, slow numpy program that follows the paper's statement of the block
(Sections 2, 4.1 and 4.4) step by step: bit-exact OCP E4M3/E5M2 encoding,
per-tensor and per-channel scales, fp64 accumulation of every contraction.
It exists so that the HIP kernels can be checked against something that can be
compared with the paper by eye.  It shares no code, tables or helpers with the
HIP path, and the product (the package with the C-ABI library) never imports
it: only the tests, the smoke check and the benchmark's CPU-baseline leg do.

``adam.py`` is the optimizer step of Section 5 with the first moment stored in
E4M3 and the second in E5M2.

Parity status of the readings the paper does not fix (formula of the
per-channel scale s_i, formula of the per-tensor scale, straight-through
gradient conventions; for the optimizer: Adam with decoupled decay, per-tensor
moment scales, update from the unrounded moments): **parity unpinned** -- they are fixed only by the
readings stated in the docstrings of ``quant.py`` and ``mlp.py``.  Everything
else is pinned by the CPU tests (closed forms, exhaustive code round trips,
exact integer brute force, fp64 autograd of the unquantized function).
"""
from . import fp8, quant, swiglu, gemm, mlp, adam, scaling, infer  # noqa: F401
