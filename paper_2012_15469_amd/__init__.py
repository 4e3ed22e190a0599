"""CADA hot path for MI355X: C-ABI library libcada.so plus a thin ctypes binding.

Importing this package does not load the library; ``binding`` does, and fails
loudly if the library has not been built (``python -m paper_2012_15469_amd.build``).
"""
