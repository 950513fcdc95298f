"""Seeded synthetic inputs and the user programs (traces) of the benchmark
configurations.

This package holds *inputs to the method* only: random data generators and
tensor programs written against an abstract tensor API (any object with
methods ``mul``, ``add``, ``sum``, ``matmul`` ...).  It contains none of the
method's own arithmetic, recording, hashing, lowering or kernels, so it can be
handed both to the HIP library's front end and to the CPU oracle.
"""
