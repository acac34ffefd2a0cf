"""Seeded synthetic inputs shared by the CPU oracle tests and the HIP path.

This module holds no arithmetic of the method itself (no kernel function, no
solver step): it only draws point sets, targets, hyper-parameters and
right-hand sides with the shapes and value distributions of the paper's
regression workloads (Results section, Table 1: n from ~10^4 to ~1.3*10^6
points, d from 3 to a few hundred, whitened inputs, standardised targets).
The UCI files themselves are not used anywhere; these draws stand in for them.

All draws come from numpy's PCG64 generator in fp64 and are cast to fp32.
"""
from .configs import (Workload, make_workload, CONFIG_NAMES, rademacher,
                      base_seed, well_separated_points)

__all__ = ["Workload", "make_workload", "CONFIG_NAMES", "rademacher",
           "base_seed", "well_separated_points"]
