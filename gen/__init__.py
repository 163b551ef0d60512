"""Seeded synthetic inputs (graphs, tables, weights, upstream gradients) shared by the
tests of the CPU oracle and of the GPU path.  Holds no arithmetic of the layer."""
from . import graphs, rng, workloads  # noqa: F401
