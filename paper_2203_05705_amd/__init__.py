"""Approximate Random Dropout training GEMMs, native on AMD MI355X (gfx950).

The compute lives in ``libard.so`` (hand-written HIP behind a C ABI, see
``include/ard.h``); :mod:`paper_2203_05705_amd.binding` only marshals arguments.
Importing the package does not load the library; the first call does, and it
raises if the library has not been built.
"""
__all__ = ["binding", "workloads"]
