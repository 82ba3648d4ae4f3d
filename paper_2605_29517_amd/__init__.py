"""Fused MaxSim (late-interaction scoring) for MI355X / gfx950.

The compute path is the HIP library ``libmaxsim.so`` built from ``csrc/``; ``binding``
marshals arguments into its C ABI.  Importing this package does not load the library;
the first call does, and fails loudly when it is missing.
"""
