"""Seeded synthetic shard sets (inputs only).

This package builds the INPUTS that both the CPU oracle and the HIP library
are run on: an arena of bytes standing in for one GPU's memory, and a list of
shard views into it (dtype, shape, strides, position).  It contains none of
the method's arithmetic: no file offsets, no image, no packing.  Each side
turns a `Workload` into its own descriptor table.
"""
from .configs import (  # noqa: F401
    DTYPES,
    Shard,
    Workload,
    by_name,
    fragmentation,
    llama_rank,
    llama_7b_rank,
    llama_70b_rank,
    tiny_gpt,
)
