"""Kernel-segregated transpose convolution (arxiv 2209.03704) for MI355X / gfx950.

The compute lives in the C-ABI HIP library ``libkst.so`` (sources under
``csrc/``, declarations in ``include/kst.h``); ``binding`` marshals arguments
to it and nothing else.  ``workloads`` holds the seeded synthetic layers.
Importing the package does not load the library; the first call does, and it
raises if the library has not been built.
"""
__all__ = ["binding", "workloads", "metrics"]
