"""AoT multi-stream DAG executor for MI355X: thin Python binding over libnimble_graph.so.

``binding`` mirrors the C ABI of ``include/nimble_graph.h`` name for name (argument
marshalling only); ``runner`` registers a workload description and owns the torch
tensors (weights, arena, streams) the library borrows.
"""
from . import binding  # noqa: F401
from .runner import GraphRunner  # noqa: F401
