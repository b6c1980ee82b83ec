"""Gossip-PGA (arXiv 2105.09080) for n simulated nodes on one MI355X.

Sub-modules:
  inputs   seeded synthetic inputs and the workload table (data only)
  build    builds libgpga.so with hipcc (gfx950)
  binding  ctypes binding of the C ABI declared in include/gpga.h
  harness  torch device-memory plumbing around the binding

The binding is imported lazily so that the data generators can be used on a
machine where the library has not been built; using the method itself without
the built HIP library raises ImportError (there is no fallback).
"""
__all__ = ["inputs", "build", "binding", "harness"]
