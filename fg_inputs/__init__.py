"""Seeded synthetic inputs shared by the CPU checker and the GPU path.

Nothing here implements a step of the method; these modules only make graphs,
mini-batches, features, weights and gradient norms from a master seed.
"""
from . import rng, features, graph, sampler, workload  # noqa: F401
