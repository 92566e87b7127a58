"""Seeded synthetic workloads for the Finch selection path.

This package only *draws inputs* (prompt queries, document keys/values, lengths).
It contains none of the method's arithmetic: no softmax, no scoring, no top-r, no
gather, no schedule.  Both the CPU oracle's tests and the HIP path's tests/bench
take their inputs from here so that they see the same bytes.
"""
from .configs import (Workload, Request, WORKLOADS, get_workload, problems_of,
                      problem_seed)
from .generate import (make_problem, make_layer, to_numpy_storage, from_numpy_storage,
                       planted_positions)

__all__ = ["Workload", "Request", "WORKLOADS", "get_workload", "problems_of",
           "problem_seed", "make_problem", "make_layer", "to_numpy_storage",
           "from_numpy_storage", "planted_positions"]
