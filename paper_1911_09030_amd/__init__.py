"""Local AdaAlter (arXiv 1911.09030, Algorithm 3) hot path for AMD MI355X.

``binding`` wraps the C-ABI library built from ``csrc/``; ``workloads`` holds the
seeded synthetic inputs.  Importing the package loads nothing native; the
library is loaded on first use of ``binding`` and fails loudly if it is missing.
"""
__all__ = ["binding", "workloads"]
