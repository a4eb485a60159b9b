"""Parameter averaging across replicas (float64, NumPy).

TEST INFRASTRUCTURE ONLY - see oracle/__init__.py.

After every replica has processed its share of samples, the parameters of all
replicas are replaced by their arithmetic mean (an average, not a sum of the
changes: Sec. 3.1).  The paper redistributes the mean by starting new
processes, which rebuild their preconditioner state from the first minibatch
they see (App. B.3.2); `reset_preconditioners` reproduces that.
"""
from __future__ import annotations

import numpy as np


def average_parameters(networks, reset_preconditioners: bool = True) -> None:
    n = len(networks)
    n_layers = networks[0].n_layers
    for l in range(n_layers):
        mean = np.zeros_like(networks[0].W[l])
        for net in networks:
            mean += net.W[l]
        mean /= n
        for net in networks:
            net.W[l] = mean.copy()
    if reset_preconditioners:
        for net in networks:
            net.reset_preconditioners()


def job_learning_rate(effective_learning_rate: float, n_jobs: int) -> float:
    """Learning rate of each of `n_jobs` replicas whose parameters are averaged (Sec. 3.1): averaging dilutes
    every job's update n_jobs-fold, so the jobs' rate is the effective rate times the number of jobs."""
    if n_jobs < 1:
        raise ValueError("n_jobs must be at least 1")
    return float(effective_learning_rate) * int(n_jobs)
