"""CPU oracle for one rank's share of GEMM+reduce-scatter and all-gather+GEMM.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library and its
Python binding) may import, call or link anything in this package; only the
tests, the smoke check and the benchmark's CPU-baseline leg do.  The oracle is
deliberately plain and slow: numpy in float64, the plain definition of each
result written out (paper section 4.1 for the problem statement: an M x N x K
GEMM with an M x K first operand and a K x N second operand, 16-bit or 8-bit
inputs, wide accumulation; section 3.1.3 for reduce-scatter as the sum of the
per-rank tile contributions at the owning rank).  No blocking, fusion or
reordering.  It shares no code with the HIP path.

Every function here is pinned by tests that do not go through the function
itself (exact integer / rational brute force, closed forms, values the paper
prints, library decoders): none is "parity unpinned".
"""
from . import codec, tp_gemm, cost_model  # noqa: F401
