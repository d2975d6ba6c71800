"""Seeded synthetic inputs for LoRANN's query phase: corpora, query batches and the index arrays.

This sub-package produces *inputs only*.  It holds none of the query-phase arithmetic (routing, int8
scoring, candidate selection, re-ranking): that lives twice, independently, in the HIP library and in the
CPU oracle, and neither of those imports the other.  Both consume the arrays made here.
"""
from .workloads import Workload, WORKLOADS, get_workload
from .data import make_dataset, draw_queries
from .index_builder import build_index, random_index, IndexArrays
from .index_file import save_index, read_index

__all__ = ["Workload", "WORKLOADS", "get_workload", "make_dataset", "draw_queries", "build_index", "random_index", "save_index", "read_index", "IndexArrays"]
