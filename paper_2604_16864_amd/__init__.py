"""HieraSparse hot path for AMD MI355X: thin Python binding over the C-ABI library.

Importing the package loads nothing native; `paper_2604_16864_amd.binding.lib()`
loads `libhs.so` on first use and raises if it has not been built.
"""
__all__ = ["binding", "workloads"]
