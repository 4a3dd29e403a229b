"""CPU oracle for graph-KV attention.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 statement of what the hot path computes, written from the
paper's problem statement (Topology-Aware State Management section: every wGraph
operation node carries a precomputed KV segment; a request's KV is assembled
from the nodes on its prefix path; Eq. 7 with a zero residual).  It shares no
code with the HIP library and imports nothing from the product package.  Only
tests, the smoke check and the benchmark's cpu_baseline leg may call it.

Parity status of each function is stated in its module header.
"""
