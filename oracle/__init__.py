"""Reference oracle for the MuLoCo optimizer hot path: TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 NumPy implementation of what the GPU library computes, written
from the paper's equations (Sec. 2 "Muon", Sec. 4.1 eqs. 1-3, Algorithms 1 and 2).
It shares no code with the HIP path and must never be imported by the product
package; only the tests, the smoke check and the benchmark's CPU-baseline leg use it.

Every function here is pinned by CPU-only tests against closed forms, invariants,
textbook special cases or brute force (tests/test_oracle_*.py); there is no
"parity unpinned" function in this package.
"""
from . import storage, muon, diloco  # noqa: F401
