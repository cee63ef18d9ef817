"""Seeded synthetic inputs for isomorphic sparse collectives.

This package is the only code shared by the CPU oracle's tests and the GPU
path's tests: neighbourhood (offset list) generators, a counter-based block
content generator, and the table of benchmark workloads.  It contains none of
the method's arithmetic: nothing here knows how a torus wraps, which rank is
whose source, or what a schedule is.
"""
from .neighborhoods import (moore, von_neumann, positive_octant, shales,
                            random_distinct, stencil_block_sizes, packed_displacements)
from .blocks import (mix32, block_words, block_bytes, block_bytes_torch,
                     ALLGATHER_TWEAK, alltoall_send, allgather_send,
                     block_words_torch, alltoall_send_torch,
                     allgather_send_torch)
from .configs import CONFIGS, Workload, get_config

__all__ = [
    "moore", "von_neumann", "positive_octant", "shales", "random_distinct",
    "stencil_block_sizes", "packed_displacements",
    "mix32", "block_words", "block_bytes", "block_bytes_torch", "ALLGATHER_TWEAK", "alltoall_send", "allgather_send",
    "block_words_torch", "alltoall_send_torch", "allgather_send_torch",
    "CONFIGS", "Workload", "get_config",
]
