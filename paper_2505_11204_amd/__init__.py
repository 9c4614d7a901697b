"""RanDeS (Randomized Delta Superposition) merge / retrieve on MI355X.

The arithmetic lives in ``librandes.so`` (hand-written HIP for gfx950 behind a
C ABI, see ``include/randes.h``); :mod:`paper_2505_11204_amd.binding` only
marshals arguments.  :mod:`paper_2505_11204_amd.workloads` holds synthetic
stack shapes and seeded input generators and does not touch the library.
"""
__all__ = ["binding", "workloads", "build"]
