"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests."""
from .generators import *  # noqa: F401,F403
