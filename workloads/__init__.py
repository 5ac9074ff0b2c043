"""Seeded synthetic inputs shared by every consumer (simulators, tests, benchmark).

Holds table builders and workload recipes only; nothing here simulates.
"""
from . import laws, configs  # noqa: F401
from .configs import ALPHA, CLASSES, FLOW, GREEDY, MC, Cell, Workload  # noqa: F401
from .laws import Law, Mixture, RequestClass  # noqa: F401
