"""MI355X-native APE attention hot path (arXiv 2502.05431): a C-ABI HIP library
(``csrc/``), its thin Python binding (``binding``) and seeded synthetic
workloads (``workloads``).  Importing the package loads nothing native; the
binding loads ``libape_hip.so`` on first use and fails loudly if it is missing.
"""
__all__ = ["binding", "workloads"]
