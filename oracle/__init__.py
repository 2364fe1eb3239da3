"""CPU oracle for the replayed-routing MoE layer (arxiv 2510.11370, Section 4.1).

TEST INFRASTRUCTURE ONLY: imported by the tests, by the smoke check and by the
benchmark's cpu_baseline leg.  The GPU library never imports it, and it never
imports the GPU library.

``sparse``  - ctypes wrapper over the plain C implementation (r3_oracle.c):
              the layer by the permute -> grouped expert -> combine route.
``dense``   - NumPy float64 brute force: every expert on every token, dense
              0/1 masks, exactly as the paper's equations are written.
"""
from . import dense, sparse  # noqa: F401
