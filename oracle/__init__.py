"""Test infrastructure: the fp64 CPU oracle of the ToMA layer path (see toma_oracle.c).

Only tests, the smoke check and the benchmark's CPU-baseline leg import this package.
"""
