"""Seeded synthetic inputs (layer graphs, weights, inputs, arrivals, allocation problems).

Shared by the CPU oracle and the GPU library's tests and benchmark; contains none of
the method's arithmetic."""
from .graphs import *  # noqa: F401,F403
from .alloc_problems import *  # noqa: F401,F403
