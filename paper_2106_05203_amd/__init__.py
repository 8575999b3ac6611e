"""MI355X-native EF21 hot path: Python binding of the C-ABI library ``libef21.so``.

Importing the package loads nothing; the HIP library is opened on first use of
``paper_2106_05203_amd.binding`` and a missing library is an error, never a fallback.
"""
__all__ = ["binding", "workloads"]
