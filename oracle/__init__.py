"""CPU oracle for the DVM hot path.  TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may import
this package.  It shares no code with the HIP path (``paper_2603_24239_amd/``) and imports nothing
from it; the product never calls it.

  interp.py  -- plain per-op eager interpreter of an operator program (float64, NumPy): every op is a
               full pass that materialises its result, no tiling, no fusion (the fused VM must compute
               exactly the unfused definition: Section 5.1, pattern-based fusion only moves
               intermediates from global to local memory).
  tiling.py  -- brute-force statement of the tile-size cost model (Section 4.2, "Shape tiling") and of
               the tile-to-core assignment of Algorithm 2.
"""
