"""Seeded synthetic inputs for the ParaRNN hot path.

This package holds only the random-number generator and the shapes / value
distributions of the benchmark configurations.  It contains none of the
method's arithmetic: both the CPU oracle's tests and the GPU path's tests
draw their bytes from here, and neither side's code is imported.
"""
from .rng import uniform01, normal, uniform_sym
from .configs import ALL_CONFIGS, CONFIGS, EXTRA_CONFIGS, Workload, make_inputs, cell_dims

__all__ = ["uniform01", "normal", "uniform_sym", "ALL_CONFIGS", "CONFIGS", "EXTRA_CONFIGS", "Workload",
           "make_inputs", "cell_dims"]
