"""Python face of the CPU oracle (test infrastructure, never the product path).

Loads oracle/libds_oracle.so (built from ds_oracle.c by `build()` below) and
offers it over `workloads.Workload` inputs; also holds `twin_pack`, a second,
independent statement of the same image written with numpy's strided views,
used only to cross-check the C loops on small inputs.

Only tests/, the smoke check and the CPU-baseline leg of bench.py may import
this module.  It imports nothing from the HIP package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ds_oracle.c")
_LIB = os.path.join(_HERE, "libds_oracle.so")

MAX_DIMS = 6
OK, BAD_ARG, BAD_ALIGN, OVERLAP, GAP, OUT_OF_IMAGE = 0, -1, -2, -3, -4, -5


class OracleShard(ctypes.Structure):
    _fields_ = [
        ("base", ctypes.c_void_p),
        ("dtype", ctypes.c_uint32),
        ("ndim", ctypes.c_uint32),
        ("shape", ctypes.c_int64 * MAX_DIMS),
        ("strides", ctypes.c_int64 * MAX_DIMS),
        ("tensor_id", ctypes.c_uint64),
        ("file_offset", ctypes.c_uint64),
    ]


def build(force: bool = False) -> str:
    """Compile ds_oracle.c with gcc into libds_oracle.so (plain C, -O2)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.run(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fPIC", "-shared", "-pthread",
                        "-o", _LIB, _SRC], check=True)
    return _LIB


_lib = None


def bind(path: str) -> ctypes.CDLL:
    """Load a build of the oracle and declare its signatures."""
    L = ctypes.CDLL(path)
    P = ctypes.POINTER(OracleShard)
    L.dso_itemsize.argtypes = [ctypes.c_uint32]
    L.dso_itemsize.restype = ctypes.c_int
    L.dso_shard_bytes.argtypes = [P]
    L.dso_shard_bytes.restype = ctypes.c_int64
    L.dso_layout.argtypes = [P, ctypes.c_size_t, ctypes.c_uint64, ctypes.POINTER(ctypes.c_uint64)]
    L.dso_image_bytes.argtypes = [P, ctypes.c_size_t, ctypes.c_uint64, ctypes.POINTER(ctypes.c_uint64)]
    L.dso_check_layout.argtypes = [P, ctypes.c_size_t, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int]
    L.dso_pack.argtypes = [P, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_uint64]
    L.dso_unpack.argtypes = [P, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_uint64]
    L.dso_pack_mt.argtypes = [P, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int]
    L.dso_sizeof_shard.restype = ctypes.c_size_t
    assert L.dso_sizeof_shard() == ctypes.sizeof(OracleShard)
    return L


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        _lib = bind(_LIB)
    return _lib


def table(shards: Sequence, base_address: int):
    """Descriptor table for `workloads.Shard`-like entries whose byte_offset is
    relative to `base_address` (for the oracle: the host arena's address)."""
    n = len(shards)
    arr = (OracleShard * max(n, 1))()
    from workloads import DTYPES
    for i, s in enumerate(shards):
        d = arr[i]
        d.base = base_address + s.byte_offset
        d.dtype = DTYPES[s.dtype][0]
        d.ndim = len(s.shape)
        for j, (e, st) in enumerate(zip(s.shape, s.strides)):
            d.shape[j] = e
            d.strides[j] = st
        d.tensor_id = s.tensor_id
        d.file_offset = 0
    return arr


def layout(tab, n: int, align: int) -> int:
    total = ctypes.c_uint64(0)
    rc = lib().dso_layout(tab, n, align, ctypes.byref(total))
    if rc != OK:
        raise ValueError(f"dso_layout -> {rc}")
    return int(total.value)


def image_bytes(tab, n: int, align: int) -> int:
    total = ctypes.c_uint64(0)
    rc = lib().dso_image_bytes(tab, n, align, ctypes.byref(total))
    if rc != OK:
        raise ValueError(f"dso_image_bytes -> {rc}")
    return int(total.value)


def check_layout(tab, n: int, align: int, total: int, strict: bool = False) -> int:
    return int(lib().dso_check_layout(tab, n, align, total, 1 if strict else 0))


def pack(tab, n: int, total: int, threads: int = 1, out: Optional[np.ndarray] = None) -> np.ndarray:
    image = out if out is not None else np.empty(total, dtype=np.uint8)
    assert image.size >= total and image.dtype == np.uint8 and image.flags.c_contiguous
    if threads <= 1:
        rc = lib().dso_pack(tab, n, image.ctypes.data, total)
    else:
        rc = lib().dso_pack_mt(tab, n, image.ctypes.data, total, threads)
    if rc != OK:
        raise ValueError(f"dso_pack -> {rc}")
    return image


def unpack(tab, n: int, image: np.ndarray) -> None:
    assert image.dtype == np.uint8 and image.flags.c_contiguous
    rc = lib().dso_unpack(tab, n, image.ctypes.data, image.size)
    if rc != OK:
        raise ValueError(f"dso_unpack -> {rc}")


def pack_workload(w, threads: int = 1) -> Tuple[np.ndarray, List[int]]:
    """Canonical layout + image of a workload's host arena; returns the image
    and the offset assigned to every shard."""
    tab = table(w.shards, w.arena.ctypes.data)
    n = len(w.shards)
    total = layout(tab, n, w.align)
    image = pack(tab, n, total, threads=threads)
    return image, [int(tab[i].file_offset) for i in range(n)]


# ---------------------------------------------------------------------------
# independent twin: the same image stated with numpy views (small inputs only)
# ---------------------------------------------------------------------------

def twin_pack(w, offsets: Sequence[int], total: int) -> np.ndarray:
    """image = zeros; image[off_i : off_i + bytes_i] = bytes of the C-order copy
    of view i.  The view is rebuilt with numpy.lib.stride_tricks.as_strided over
    the arena, and numpy's own tobytes() does the element walk."""
    from numpy.lib.stride_tricks import as_strided
    from workloads import DTYPES
    image = np.zeros(total, dtype=np.uint8)
    for s, off in zip(w.shards, offsets):
        _, itemsize, npdt = DTYPES[s.dtype]
        if s.numel == 0:
            continue
        if len(s.shape) == 0:
            span = 1
        else:
            span = 1 + sum((e - 1) * st for e, st in zip(s.shape, s.strides))
        flat = w.arena[s.byte_offset:s.byte_offset + span * itemsize].view(npdt)
        view = as_strided(flat, shape=s.shape, strides=tuple(st * itemsize for st in s.strides), writeable=False)
        raw = np.frombuffer(np.ascontiguousarray(view).tobytes(), dtype=np.uint8)
        image[off:off + raw.size] = raw
    return image


def image_diff(a: np.ndarray, b: np.ndarray, block_bytes: int) -> List[int]:
    """Which blocks of two equally long byte images differ: entry k is 1 if
    bytes [k*block_bytes, (k+1)*block_bytes) differ anywhere, else 0 (the last
    block may be short).  The definition the device-side comparison for
    differential snapshots is held to (the paper's conclusions name
    differential checkpointing as future work; there is nothing to cite for how)."""
    assert a.dtype == np.uint8 and b.dtype == np.uint8 and a.size == b.size and block_bytes > 0
    return [int(bool(np.any(a[lo:lo + block_bytes] != b[lo:lo + block_bytes]))) for lo in range(0, a.size, block_bytes)]
