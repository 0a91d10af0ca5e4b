"""Block elision of an image: the oracle of the compressed-snapshot experiment (test infrastructure, never the
product path; imports nothing from the HIP package).

DataStates-LLM's conclusions name data reduction (differential checkpointing, compression) as future work and
give no method, so there is nothing in the paper to cite for HOW: the scheme below is this build's own, stated
here in plain numpy so that the device kernels can be held to it byte for byte.  **Parity unpinned against the
paper**; what pins it are its own invariants (tests/test_oracle_pins.py): decompress(compress(x)) == x, the
flags against a byte-by-byte loop, hand-made images.

Scheme.  The image is cut into blocks of `block_bytes` (the last one may be short).  A block is CONSTANT if every
16-byte unit of it equals its first unit (all-zero padding, zero-initialised optimizer moments and any periodic
fill with a period that divides 16 are of that kind); a constant block is replaced by that unit.  The compressed
form is
    keep[k]      1 if block k is stored whole, 0 if it is constant           (n_blocks entries)
    pos[k]       number of kept blocks before block k; pos[n_blocks] = total  (n_blocks + 1 entries)
    patterns[k]  the first 16 bytes of block k                                (n_blocks x 16 bytes)
    packed       the kept blocks one behind the other, each in a slot of block_bytes: block k at
                 packed[pos[k] * block_bytes ...] (the slot of a short last block is filled up to its length)
The image length is a multiple of 16 (it is a multiple of the plan's alignment)."""
from __future__ import annotations

from typing import Tuple

import numpy as np


def compress(image: np.ndarray, block_bytes: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray]:
    """(keep, pos, patterns, packed) of a uint8 image; packed has exactly pos[-1] slots."""
    assert image.dtype == np.uint8 and image.size % 16 == 0 and block_bytes % 16 == 0 and block_bytes > 0
    n_blocks = -(-image.size // block_bytes)
    keep = np.zeros(n_blocks, dtype=np.uint32)
    pos = np.zeros(n_blocks + 1, dtype=np.uint32)
    patterns = np.zeros((n_blocks, 16), dtype=np.uint8)
    slots = []
    for k in range(n_blocks):
        block = image[k * block_bytes:(k + 1) * block_bytes]
        units = block.reshape(-1, 16)
        patterns[k] = units[0]
        keep[k] = 0 if np.all(units == units[0]) else 1
        pos[k + 1] = pos[k] + keep[k]
        if keep[k]:
            slot = np.zeros(block_bytes, dtype=np.uint8)
            slot[:block.size] = block
            slots.append(slot)
    packed = np.concatenate(slots) if slots else np.zeros(0, dtype=np.uint8)
    return keep, pos, patterns, packed


def decompress(keep: np.ndarray, pos: np.ndarray, patterns: np.ndarray, packed: np.ndarray, nbytes: int,
               block_bytes: int) -> np.ndarray:
    """The image back from its compressed form."""
    n_blocks = -(-nbytes // block_bytes)
    assert keep.size == n_blocks and pos.size == n_blocks + 1
    out = np.empty(nbytes, dtype=np.uint8)
    for k in range(n_blocks):
        lo = k * block_bytes
        length = min(block_bytes, nbytes - lo)
        if keep[k]:
            at = int(pos[k]) * block_bytes
            out[lo:lo + length] = packed[at:at + length]
        else:
            out[lo:lo + length] = np.tile(patterns[k].reshape(16), length // 16)
    return out


def compressed_bytes(keep: np.ndarray, block_bytes: int) -> int:
    """Bytes that have to leave the device: the kept blocks, one 16-byte pattern and one flag per block."""
    return int(keep.sum()) * block_bytes + keep.size * (16 + 4)
