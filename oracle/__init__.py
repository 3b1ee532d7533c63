"""CPU oracle for the exact int8 convolution and its RNS-Winograd stages.

TEST INFRASTRUCTURE ONLY.  Only the test-suite, the smoke check and the
benchmark's cpu_baseline leg may import this package; the product package
never does, and this package never imports the product.  Inputs are passed in
as numpy arrays; nothing here draws random numbers.

  direct   -- the plain definition (C, seven nested loops): `direct_conv2d`,
              plus the shift/clamp re-quantisation and 2x2 max-pool that glue
              the layers of the 13-layer stack workload together.
  rnswino  -- the paper's algorithm step by step in numpy int64 / Fractions
              (transform matrices, residues, per-stage tensors, mixed-radix
              back-conversion), used for stage-level parity.
"""
from .direct import direct_conv2d, requant_shift_clamp, maxpool2x2, build_direct, num_threads  # noqa: F401
from . import rnswino  # noqa: F401
