"""CommFuse rank-step hot path for AMD MI355X (gfx950).

The compute lives in ``libcommfuse.so`` (hand-written HIP, C ABI declared in
``include/commfuse.h``); :mod:`paper_2604_24013_amd.binding` marshals arguments
to it and nothing else.  Importing this package does not load the library;
the binding loads it on first use and raises if it has not been built.
"""
__all__ = ["binding", "inputs", "build"]
