"""CPU oracle for the packed multi-LoRA linear layer.  TEST INFRASTRUCTURE ONLY.

Two independent writings of the same definition (paper sections 2.1, 2.4 and the four gradient
cases of appendix C.2), both computing in fp64:

* ``loops``  - plain C scalar loops (``plora_oracle.c``), callable per token row and per adapter,
  so that sampled outputs of full-size problems can be computed one by one;
* ``matmul`` - the same formulas with numpy's fp64 matrix product as the step, fast enough for
  whole tensors of the larger configurations.

``adamw`` holds the per-adapter optimizer step that follows the backward pass (fp64, element by
element).  ``nf4`` holds the 4-bit storage format of a quantised base weight (the layer on such a
weight is the layer above on its dequantised values).  ``planner`` holds the scheduling side of the
paper (memory model, packing of one job by enumeration, DTM, job planner, tail bound).

Nothing here imports, or is imported by, the HIP library or its binding.  Only the tests, the
smoke check and the benchmark's ``cpu_baseline`` leg may use this package.
"""
from .problem import Problem  # noqa: F401
from . import adamw, loops, matmul, nf4, planner  # noqa: F401
