"""Shared-prompt attention (Section 4.3 of arXiv 2511.18871) for AMD MI355X.

`binding` holds the ctypes wrappers of the C-ABI library; `workloads` the seeded
synthetic inputs.  Importing the package loads nothing heavy."""
__all__ = ["binding", "workloads", "build"]
