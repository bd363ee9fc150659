"""Seeded synthetic gradient streams for the rTop-k hot path.

This package holds input generators only: it draws random gradient vectors
with the sizes and value structure of the workloads the method was evaluated
on (image-classification and language-model gradients; Section IV), and it
computes nothing the method itself defines beyond the integer ceilings that
turn the (r/d, k/d) percentages of a configuration into counts. It is
imported by the tests, the benchmark and the smoke check; both the CPU oracle
and the HIP library receive its output as plain arrays.
"""
from .gradients import CONFIGS, Workload, ceil_fraction, philox_seed_for_worker

__all__ = ["CONFIGS", "Workload", "ceil_fraction", "philox_seed_for_worker"]
