"""Seeded synthetic inputs shared by the oracle-side tests and the HIP-side harness.

Holds no arithmetic of the method: only shapes, seeds and raw random draws.
"""
from .generators import *  # noqa: F401,F403
