"""Seeded synthetic inputs shared by the CPU oracle, the HIP path, the tests and the bench.

This package only draws numbers and lays them out (prompts, target lengths,
weights, page tables, attention operands).  None of the rollout method's
arithmetic (forward pass, attention, scheduling) lives here.
"""
from .gen import *  # noqa: F401,F403
