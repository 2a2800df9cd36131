"""On-the-fly operation batching on MI355X: Python binding over the C-ABI library.

The HIP library is loaded on first use (see `binding`); importing the package
itself needs no GPU so that workload generators can be used on a CPU-only host.
"""
__all__ = ["workloads", "binding"]
