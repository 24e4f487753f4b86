"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP library's
tests and benchmark.  Generators only: nothing of the layers' arithmetic."""
from . import graphs, configs  # noqa: F401
from .configs import make, NAMES  # noqa: F401
