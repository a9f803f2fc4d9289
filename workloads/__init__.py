"""Program descriptions and seeded inputs shared by the oracle, the HIP binding, the tests and the bench.

Data only: no combinator is evaluated and no partition is chosen in this package.
"""
from .graph import Graph, Node, single_pass
from .configs import Workload, build, BUILDERS, SMALL, SEED0

__all__ = ["Graph", "Node", "single_pass", "Workload", "build", "BUILDERS", "SMALL", "SEED0"]
