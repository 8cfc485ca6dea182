"""CPU oracle for the RSR++ vector x binary/ternary-matrix product.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The HIP library never imports, links or calls
anything in this package, and nothing here imports the HIP package.

Two layers:

* ``oracle.dense``  - the plain definition ``out[b][c] = sum_r v[b][r]*A[r][c]``
  (Section 2.2, Problems 1 and 2) as straightforward C loops (``rsr_oracle.c``),
  float64 accumulation for float activations and int64 for int8 activations.
  This is what the GPU result is compared against.
* ``oracle.steps``  - the paper's intermediate objects written out in its own
  notation (ternary split, k-column blocks, binary row order, Bin_[k], full
  segmentation, segmented sums, the RSR block product and the RSR++ fold), used
  to check the index tables the library builds and to pin the readings of the
  paper that the build relies on.
"""
from . import dense, steps  # noqa: F401
