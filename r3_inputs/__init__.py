"""Seeded synthetic workloads for the replay-evaluation path (no arithmetic of the method)."""
from .configs import *  # noqa: F401,F403
