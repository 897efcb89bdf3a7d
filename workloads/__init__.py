"""Seeded synthetic inputs and the named workload configurations.

This module produces *inputs only*: datasets, initial points and hyper-parameter
records.  It contains none of the method's arithmetic (no gradients, no updates,
no averaging, no index sampling) so that both the CPU oracle and the HIP path
can be fed identical bytes without sharing any of the code under test.
"""
from .configs import Workload, WORKLOADS, get_workload  # noqa: F401
from .synth import (  # noqa: F401
    make_lsq_data,
    make_gmm_data,
    make_x0,
    make_inputs,
    param_count,
)
