"""Batched Forward Prune (Algorithm 1 of the Dragon paper, arXiv 1707.08265) on AMD CDNA4.

The package is a thin binding over ``libdgn.so`` (HIP kernels + C ABI, see ``include/dgn.h``).
Build the library first: ``python __graft_entry__.py`` at the repository root (or ``python
paper_1707_08265_amd/build.py``): the package cannot be imported without it.
"""
from .binding import *  # noqa: F401,F403
from .binding import (DeviceGraph, PruneBuffers, BackwardPruneBuffers, InplaceBuffers, ReadoutBuffers, TransactionCache,
                      DgnError, EXPORTS,
                      LIB_PATH)  # noqa: F401
