"""Seeded synthetic workloads: network graphs, rollout patterns, weights and
input frame sequences.  Holds no part of the rollout arithmetic; it is the only
code shared by the CPU oracle's tests and the GPU path's tests."""
from .graphs import *  # noqa: F401,F403
from .inputs import make_weights, make_inputs, make_case  # noqa: F401
