"""Seeded synthetic inputs (graphs, budgets, candidate batches).

Shared by the tests of the CPU oracle and of the HIP library; holds no
arithmetic of the evaluated method and imports neither of them.
"""
from .graphs import Graph, graph_from_edges  # noqa: F401
from .workloads import Workload, make_workload, workload_from_graph  # noqa: F401
from .device import DeviceWorkload, stream_read  # noqa: F401,E402
