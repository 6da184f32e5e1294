"""CPU oracle for fused-subgraph execution and error scoring.

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's CPU-baseline leg, never by the product path.
"""
