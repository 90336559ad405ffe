"""CPU oracle for the stencil skeleton and its workgroup-size sweep.

TEST INFRASTRUCTURE ONLY: imported by tests/, by `__graft_entry__.smoke()` and by the
`cpu_baseline` leg of bench.py.  Nothing in the product package imports it, and it imports
nothing from the product package.

  oracle.stencil  - the stencil itself (plain C loops in stencil_oracle.c, called via ctypes)
  oracle.tuning   - the host-side definitions around the sweep: size enumeration, legality
                    (Eq. 1), oracle size (Eq. 3), performance / speedup metrics (Section 7),
                    the NearestNeighbour fallback (Algorithm 1) and the 1-NN classifier.
"""
from . import stencil, tuning  # noqa: F401
