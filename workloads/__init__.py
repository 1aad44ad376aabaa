"""Seeded synthetic inputs for the five fused-operator workloads.

This package only draws random inputs and names the workloads; it contains none
of the method's arithmetic.  Both the CPU oracle's tests and the GPU library's
tests/benchmark take their inputs from here.
"""
from .gen import (BASE_SEED, seed_for, dense_uniform, dense_normal, csr_bernoulli,  # noqa: F401
                  csr_fixed_per_row, csr_skewed)
from .configs import WORKLOADS, make_workload  # noqa: F401
