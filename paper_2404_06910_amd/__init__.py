"""MI355X-native hot path of superposition prompting: thin Python binding over libsp.so.

The package only marshals arguments; every step of the path runs in the HIP kernels of
libsp.so (see include/sp.h for the C ABI).  Importing the package does not load the library;
the first use does, and fails loudly if it has not been built.
"""
from .binding import (SpError, Context, Plan, lib, lib_path, equilibrium_positions, SP_F32, SP_BF16,
                      SALIENCY_SUM, SALIENCY_MEAN)

__all__ = ["SpError", "Context", "Plan", "lib", "lib_path", "equilibrium_positions", "SP_F32", "SP_BF16",
           "SALIENCY_SUM", "SALIENCY_MEAN"]
