"""Seeded synthetic inputs (graphs, objective data, schedules) shared by the
oracle-side tests and the GPU-side tests.  Holds no arithmetic of the method."""
from . import configs, graphs, problems, schedule  # noqa: F401
