"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

Holds no arithmetic of the training step: only graph shapes, id draws and the
workload table.  The public datasets the paper trains on (Table 1) are not
available offline; these generators produce stand-ins with the same sizes,
degree skew and relation mix.
"""
from .configs import CONFIGS, Workload, get_workload      # noqa: F401
from .graphs import make_graph, make_tables, zipf_ids     # noqa: F401
