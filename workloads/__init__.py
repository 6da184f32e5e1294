"""Seeded synthetic workloads: input tensors and op-DAGs in text form.

Holds no arithmetic of the method; both the oracle and the HIP library read
what this package emits.
"""
