"""CPU oracle for the triplet interaction block (TEST INFRASTRUCTURE ONLY).

A plain, slow, fp64 implementation of what the HIP library computes, written
from the paper's definitions (Sec. 3.1 graph and triplet definition, Sec. 3.3
message update equation, Sec. 3.4 bilinear variant, Sec. 3.2 forces as the
negative energy gradient).  It shares no code with the HIP path and is only
ever imported by the tests, by the smoke check and by the benchmark's CPU
baseline leg.  The product path never routes through it.

Modules
  graph   radius graph and triplet lists (numpy; fp32 distance predicate)
  basis   envelope, radial / spherical / Gaussian bases (torch fp64)
  block   interaction blocks, variants D (Hadamard) and G (bilinear) (torch fp64)
  energy  per-atom energy head, energy and forces by automatic differentiation
"""
