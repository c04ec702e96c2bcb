"""fp64 CPU oracle for the Metis split-FP4 linear path.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this
package; only tests, the smoke check and the benchmark's CPU-baseline leg do.
It shares no code with the HIP kernels: every function here is written from
the paper's definitions (section / equation cited per function) in plain numpy
fp64, without blocking, fusion or reordering.

Modules
  rng        Philox4x32-10 counter-based generator, the stratified row sampler
             and the Gaussian test matrix (Sec. 3.1).
  quant      NVFP4 block quantizer: E2M1 codes, E4M3 block scales (Sec. 2.3,
             App. C.1).
  decompose  sampled randomized SVD, broadcast, split A = U S V^T + R
             (Sec. 3.1, 3.2).
  hadamard   16-point random Hadamard rotation in front of the stochastic quantizer (the
             comparison recipe of Sec. 4.3).
  mx         MXFP4 quantizer of the microscaling family (Sec. 2.3 names it beside NVFP4).
  linear     fprop / dgrad / wgrad on split-quantized operands (Eq. 2, Eq. 3
             and the W_R gradient listed after it).

Parity pins (tests/test_oracle_*.py): every function in these modules is pinned
to something other than itself; none is "parity unpinned".
"""
