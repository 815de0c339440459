"""CPU oracle for the Shfl-BW hot path.  TEST INFRASTRUCTURE ONLY.

Only ``tests/``, the smoke check and the benchmark's CPU-baseline leg may
import this package.  The product (the HIP library and its binding) never
does, and this package never imports the product.

Two independent statements of the same result live here:

* ``oracle.c_oracle`` - plain C loops over kept weights (double accumulators),
  compiled with gcc; this is the one timed as the CPU baseline.
* ``oracle.definition`` - the definition written with numpy primitives in
  float64 (masked ``matmul``; explicit unfold for convolution), plus the
  logical vector-wise format of the paper's offline step (a).

Parity status: every function is pinned by the CPU tests in
``tests/test_oracle_pins.py`` (brute force on tiny inputs, exact integer
cases, dense special case against ``numpy.matmul``, permutation invariance,
delta-kernel closed forms, library convolution).  The paper prints no worked
numeric example for this path (its examples are in figures), so no pin is a
value taken from the paper.
"""
