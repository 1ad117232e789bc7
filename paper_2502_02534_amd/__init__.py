"""Shared-prefix decode attention and token sampling for MI355X (gfx950).

The compute lives in a C-ABI shared library built from csrc/ (HIP); `binding`
marshals arguments to it.  Importing this package does not load the library;
the first call does, and raises if it has not been built.
"""
__all__ = ["binding", "workloads"]
