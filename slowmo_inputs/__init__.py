"""Seeded synthetic inputs shared by the tests, the benchmark and the oracle's
callers: tensor-shape lists, workload definitions and a counter-based value
generator (NumPy on the host, one HIP kernel on the device).  Nothing in this
package performs any step of the optimizer."""
from . import generator, shapes, workloads  # noqa: F401
