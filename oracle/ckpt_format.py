"""CPU oracle of the checkpoint FILE (test infrastructure, never the product path).

States, in plain Python, what a checkpoint file holds (DataStates-LLM
Sec. V-A5): (1) the tensors at the offsets fixed in advance, i.e. the image at
the head of the file; (2) the chunks of serialized objects appended behind the
tensors in the order they arrive; (3) a metadata trailer written last, from
which both can be found again.  The paper gives the three rules and no byte
encoding; the encoding written out here is this build's reading of them and is
what the library's header documents.  **Parity unpinned** against the paper
for the encoding itself; what the tests pin is the three rules (the tensor
region is the image, objects reassemble, everything is found from the end of
the file), a hand-written file, the checksum's textbook check value, and that
damage is detected.

Only tests/, the smoke check and bench.py's CPU leg may import this module.
It imports nothing from the HIP package.

Layout (little-endian):
    [0, T)           tensor region
    [T, E)           object log; a chunk of n bytes occupies round_up(n, 8)
    [E, ...)         trailer: 80-byte tensor entries, 32-byte chunk entries
    last 64 bytes    footer
"""
from __future__ import annotations

import struct
import zlib
from typing import Dict, List, Sequence, Tuple

MAGIC = b"DSCKPT01"
VERSION = 1
MAX_DIMS = 6

TensorEntry = Tuple[int, int, Tuple[int, ...], int, int]  # tensor_id, dtype code, shape, file_offset, nbytes


class FormatError(ValueError):
    pass


def build_file(align: int, image: bytes, tensors: Sequence[TensorEntry],
               appends: Sequence[Tuple[int, bytes]]) -> bytes:
    """The whole file as bytes.  `appends` are (object_id, chunk) in the order
    in which they were appended to the log."""
    T = len(image)
    if T % align:
        raise FormatError("image length is not a multiple of the alignment")
    out = bytearray(image)
    chunks: List[Tuple[int, int, int, int]] = []      # object_id, seq, offset, length
    seen: Dict[int, int] = {}
    for object_id, data in appends:
        seq = seen.get(object_id, 0)
        seen[object_id] = seq + 1
        chunks.append((object_id, seq, len(out), len(data)))
        out += data
        out += b"\0" * (-len(data) % 8)
    E = len(out)
    trailer = bytearray()
    for tensor_id, dtype, shape, off, nbytes in tensors:
        dims = tuple(shape) + (0,) * (MAX_DIMS - len(shape))
        trailer += struct.pack("<QII6QQQ", tensor_id, dtype, len(shape), *dims, off, nbytes)
    for c in sorted(chunks):                          # by (object_id, seq)
        trailer += struct.pack("<4Q", *c)
    footer = MAGIC + struct.pack("<IIQQQQQI", VERSION, 0, align, T, E, len(tensors), len(chunks),
                                 zlib.crc32(bytes(trailer)))
    footer += struct.pack("<I", zlib.crc32(footer))
    assert len(footer) == 64
    return bytes(out + trailer + footer)


def parse_file(blob: bytes) -> dict:
    """Inverse of build_file: the layout numbers, the tensor entries, the
    objects reassembled {object_id: bytes}, and the tensor region."""
    if len(blob) < 64:
        raise FormatError("shorter than a footer")
    f = blob[-64:]
    if f[:8] != MAGIC:
        raise FormatError("magic")
    version, flags, align, T, E, n, m, crc_t = struct.unpack("<IIQQQQQI", f[8:60])
    if struct.unpack("<I", f[60:])[0] != zlib.crc32(f[:60]):
        raise FormatError("footer checksum")
    if version != VERSION or flags != 0:
        raise FormatError("version")
    if E + 80 * n + 32 * m + 64 != len(blob) or T > E or T % align or E % 8:
        raise FormatError("bounds")
    trailer = blob[E:len(blob) - 64]
    if zlib.crc32(trailer) != crc_t:
        raise FormatError("trailer checksum")
    tensors = []
    for i in range(n):
        tid, dtype, ndim, *rest = struct.unpack_from("<QII6QQQ", trailer, 80 * i)
        shape, off, nbytes = tuple(rest[:ndim]), rest[6], rest[7]
        if off % align or off + nbytes > T:
            raise FormatError("tensor outside the tensor region")
        tensors.append((tid, dtype, shape, off, nbytes))
    objects: Dict[int, bytearray] = {}
    last = None
    for k in range(m):
        oid, seq, off, ln = struct.unpack_from("<4Q", trailer, 80 * n + 32 * k)
        if off < T or off + ln > E:
            raise FormatError("chunk outside the log")
        if last is not None and (oid, seq) <= last:
            raise FormatError("chunk order")
        if seq != (last[1] + 1 if last is not None and last[0] == oid else 0):
            raise FormatError("chunk numbering")
        last = (oid, seq)
        objects.setdefault(oid, bytearray()).extend(blob[off:off + ln])
    return {"align": align, "tensor_bytes": T, "log_end": E, "n_chunks": m, "tensors": tensors,
            "objects": {k: bytes(v) for k, v in objects.items()}, "image": blob[:T]}


# ---- one shard table, several files --------------------------------------------------------------
# A rank writes its checkpoint as several files (DataStates-LLM Sec. VI-D: 20 for a 7B rank); each
# shard of the rank's table names the file it belongs to.  Every file is a checkpoint file as above,
# built from the shards that name it; the rank's ONE image is the files' tensor regions one behind
# the other, in file order.  Parity unpinned against the paper, which states the file count only.

def rank_files(sizes: Sequence[int], file_of: Sequence[int], n_files: int, align: int):
    """Where every shard goes when one table feeds `n_files` files.

    Inside its file a shard sits at the next multiple of `align` behind the shard of the same file
    that precedes it in the table (the canonical layout, file by file).  Returns
    (offset_in_file per shard, tensor-region length per file, where each region starts in the image)."""
    if len(sizes) != len(file_of):
        raise FormatError("one file index per shard")
    at = [0] * n_files
    offs = []
    for size, f in zip(sizes, file_of):
        if not 0 <= f < n_files:
            raise FormatError("file index out of range")
        offs.append(at[f])
        at[f] += size + (-size % align)
    begins, run = [], 0
    for f in range(n_files):
        begins.append(run)
        run += at[f]
    return offs, at, begins


def build_rank_files(align: int, image: bytes, tensors: Sequence[TensorEntry], file_of: Sequence[int],
                     n_files: int, appends: Sequence[Sequence[Tuple[int, bytes]]]) -> List[bytes]:
    """The files of one rank.  `image` is the rank's whole image, `tensors` the table in table order
    with offsets INSIDE each shard's own file, appends[f] the object chunks of file f."""
    _, regions, begins = rank_files([t[4] for t in tensors], file_of, n_files, align)
    if len(image) != sum(regions):
        raise FormatError("image length is not the sum of the regions")
    return [build_file(align, image[begins[f]:begins[f] + regions[f]],
                       [t for t, g in zip(tensors, file_of) if g == f], appends[f])
            for f in range(n_files)]
