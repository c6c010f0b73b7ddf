"""MI355X-native subgraph GNN training for graph combinatorial optimisation.

Sub-modules:
  binding  -- ctypes binding of the C-ABI device library (libgco.so)
  build    -- compiles the HIP sources for gfx950
  inputs   -- seeded synthetic graphs, partition ids and initial parameters

Importing the package loads nothing native; ``binding`` loads the device
library on first use and raises if it is missing.
"""
__all__ = ["binding", "build", "inputs"]
