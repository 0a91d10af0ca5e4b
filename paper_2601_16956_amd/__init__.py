"""Thin Python binding of libdatastates_hip.so (argument marshalling only).

Every function has the name of the C entry point it calls (include/datastates.h)
and does nothing but convert arguments, call it, and turn a negative return
code into `DsError`.  All of the method runs in the HIP library; if the library
has not been built the import fails loudly -- there is no fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdatastates_hip.so")

DS_MAX_DIMS = 6
DS_F32, DS_BF16, DS_F16, DS_I64, DS_U8 = 0, 1, 2, 3, 4
DS_OK, DS_NOT_READY, DS_EOF = 0, 1, 2
DS_EINVAL, DS_EALIGN, DS_EOVERLAP, DS_EGAP, DS_ERANGE, DS_ENOMEM, DS_EHIP, DS_EBUSY, DS_ESTATE, DS_EIO = (
    -1, -2, -3, -4, -5, -6, -7, -8, -9, -10)
DS_EFORMAT = -11
DS_EFAULT = -12
DS_ETOOBIG = -13
DS_PACK_NOALLOC_TABLE_BYTES = 4 << 20
DS_FILE_DIRECT, DS_FILE_SYNC, DS_FILE_URING = 1, 2, 4
DS_PLAN_STRICT, DS_PLAN_HOST_ONLY, DS_PLAN_CHECK_MEMORY = 1, 2, 4
DS_ENGINE_AUTO_RELEASE, DS_ENGINE_TRACE = 1, 2

# every symbol include/datastates.h declares
EXPORTS = [
    "ds_itemsize", "ds_layout_assign", "ds_plan_create", "ds_plan_destroy", "ds_plan_info", "ds_plan_shard",
    "ds_pack", "ds_unpack", "ds_engine_create", "ds_engine_destroy", "ds_snapshot_async",
    "ds_event_wait_on_stream", "ds_event_wait_captured", "ds_event_query", "ds_event_wait",
    "ds_snapshot_next_chunk", "ds_snapshot_release_chunk", "ds_event_stats", "ds_event_destroy",
    "ds_strerror", "ds_last_hip_error", "ds_config_set", "ds_config_get", "ds_copy_probe",
    "ds_restore_begin", "ds_restore_next_slot", "ds_restore_submit",
    "ds_flush_start", "ds_flush_wait", "ds_restore_from_file", "ds_last_errno",
    "ds_plan_shard_shape", "ds_ckpt_create", "ds_ckpt_flush_snapshot", "ds_ckpt_write_region", "ds_ckpt_append",
    "ds_ckpt_finish", "ds_ckpt_open", "ds_ckpt_close", "ds_ckpt_layout_info", "ds_ckpt_tensor_info",
    "ds_ckpt_object_at", "ds_ckpt_object_read", "ds_ckpt_matches_plan", "ds_ckpt_restore", "ds_event_trace",
    "ds_image_diff", "ds_pack_noalloc", "ds_image_compress",
    "ds_plan_create_files", "ds_layout_assign_files", "ds_plan_file", "ds_plan_shard_file", "ds_flush_start_files",
    "ds_restore_from_files", "ds_ckpt_create_part", "ds_ckpt_flush_snapshot_parts", "ds_ckpt_matches_plan_part",
    "ds_ckpt_restore_parts", "ds_ckpt_append_from",
]


class ds_shard_desc(ctypes.Structure):
    _fields_ = [
        ("base", ctypes.c_void_p),
        ("dtype", ctypes.c_uint32),
        ("ndim", ctypes.c_uint32),
        ("shape", ctypes.c_int64 * DS_MAX_DIMS),
        ("strides", ctypes.c_int64 * DS_MAX_DIMS),
        ("tensor_id", ctypes.c_uint64),
        ("file_offset", ctypes.c_uint64),
    ]


class ds_plan_stats(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint64) for n in (
        "total_bytes", "payload_bytes", "n_shards", "n_tiles", "n_chunks", "chunk_bytes", "n_strided", "align",
        "n_general_chunks", "n_files")]


ds_chunk_provider = ctypes.CFUNCTYPE(ctypes.c_int, ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p),
                                     ctypes.POINTER(ctypes.c_uint64))


class ds_engine_opts(ctypes.Structure):
    _fields_ = [
        ("host_ring_bytes", ctypes.c_uint64),
        ("d2h_chunk_bytes", ctypes.c_uint64),
        ("stage_slot_bytes", ctypes.c_uint64),
        ("stage_slots", ctypes.c_uint32),
        ("pack_grid_limit", ctypes.c_uint32),
        ("flags", ctypes.c_uint32),
        ("copy_streams", ctypes.c_uint32),
        ("first_launch_bytes", ctypes.c_uint64),
    ]


class ds_snapshot_stats(ctypes.Structure):
    _fields_ = [
        ("image_bytes", ctypes.c_uint64),
        ("payload_bytes", ctypes.c_uint64),
        ("n_pack_launches", ctypes.c_uint32),
        ("n_copies", ctypes.c_uint32),
        ("pack_ms", ctypes.c_double),
        ("copy_ms", ctypes.c_double),
        ("capture_ms", ctypes.c_double),
        ("total_ms", ctypes.c_double),
        ("submit_host_ms", ctypes.c_double),
    ]


class ds_trace_rec(ctypes.Structure):
    _fields_ = [
        ("kind", ctypes.c_uint32),
        ("index", ctypes.c_uint32),
        ("file_off", ctypes.c_uint64),
        ("len", ctypes.c_uint64),
        ("begin_ms", ctypes.c_double),
        ("end_ms", ctypes.c_double),
    ]


class ds_ckpt_layout(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint64) for n in (
        "align", "tensor_bytes", "log_end", "n_tensors", "n_chunks", "n_objects", "file_bytes")]


class ds_ckpt_tensor(ctypes.Structure):
    _fields_ = [
        ("tensor_id", ctypes.c_uint64),
        ("dtype", ctypes.c_uint32),
        ("ndim", ctypes.c_uint32),
        ("shape", ctypes.c_int64 * DS_MAX_DIMS),
        ("file_offset", ctypes.c_uint64),
        ("nbytes", ctypes.c_uint64),
    ]


class DsError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = _lib.ds_strerror(code).decode()
        if code == DS_EHIP:
            msg += f" [hipError {_lib.ds_last_hip_error()}]"
        if code == DS_EIO:
            msg += f" [errno {_lib.ds_last_errno()}]"
        super().__init__(f"{where}: {msg} ({code})")


def hip_runtime_in_use() -> List[str]:
    """Paths of the HIP / HSA runtime libraries mapped into this process."""
    try:
        with open("/proc/self/maps") as f:
            return sorted({ln.split()[-1] for ln in f if "libamdhip64" in ln or "libhsa-runtime64" in ln})
    except OSError:
        return []


def kernel_source_digest() -> str:
    """SHA-256 (first 16 hex digits) over the kernel sources; a counter profile names the digest it was taken
    with, so that a reader of a measurement can tell whether the profile still describes the kernels in use."""
    import hashlib
    h = hashlib.sha256()
    for name in ("ds_kernels.hip", "ds_splice.h", "ds_internal.h"):
        with open(os.path.join(_HERE, "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def _load() -> ctypes.CDLL:
    # One HIP runtime per process.  The PyTorch wheel bundles its own copy of
    # libamdhip64 (soname libamdhip64.so.7, looked up by torch under the name
    # libamdhip64.so); if this library were loaded first it would pull in the
    # system copy and torch would then load a SECOND runtime, after which
    # streams and pointers could not be shared.  Loading torch first makes the
    # loader resolve this library's libamdhip64.so.7 to the copy torch brought.
    import torch  # noqa: F401
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -m paper_2601_16956_amd.build, or "
            "__graft_entry__.build()).  There is no CPU fallback.")
    L = ctypes.CDLL(LIB_PATH)
    vp, u64, u32, sz = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_size_t
    P = ctypes.POINTER
    sig = {
        "ds_itemsize": ([u32], ctypes.c_int),
        "ds_layout_assign": ([P(ds_shard_desc), sz, u64, P(u64)], ctypes.c_int),
        "ds_plan_create": ([P(ds_shard_desc), sz, u64, u32, P(vp)], ctypes.c_int),
        "ds_plan_destroy": ([vp], ctypes.c_int),
        "ds_plan_info": ([vp, P(ds_plan_stats)], ctypes.c_int),
        "ds_plan_shard": ([vp, sz, P(u64), P(u32), P(u64), P(u64)], ctypes.c_int),
        "ds_pack": ([vp, vp, u64, u64, vp], ctypes.c_int),
        "ds_unpack": ([vp, vp, u64, u64, vp], ctypes.c_int),
        "ds_pack_noalloc": ([vp, vp, u64, u64, vp], ctypes.c_int),
        "ds_engine_create": ([P(ds_engine_opts), P(vp)], ctypes.c_int),
        "ds_engine_destroy": ([vp], ctypes.c_int),
        "ds_snapshot_async": ([vp, vp, vp, P(vp)], ctypes.c_int),
        "ds_event_wait_on_stream": ([vp, vp], ctypes.c_int),
        "ds_event_wait_captured": ([vp], ctypes.c_int),
        "ds_event_query": ([vp], ctypes.c_int),
        "ds_event_wait": ([vp], ctypes.c_int),
        "ds_snapshot_next_chunk": ([vp, P(vp), P(u64), P(u64)], ctypes.c_int),
        "ds_snapshot_release_chunk": ([vp, vp], ctypes.c_int),
        "ds_event_stats": ([vp, P(ds_snapshot_stats)], ctypes.c_int),
        "ds_event_destroy": ([vp], ctypes.c_int),
        "ds_strerror": ([ctypes.c_int], ctypes.c_char_p),
        "ds_last_hip_error": ([], ctypes.c_int),
        "ds_config_set": ([ctypes.c_char_p, u64], ctypes.c_int),
        "ds_config_get": ([ctypes.c_char_p, P(u64)], ctypes.c_int),
        "ds_copy_probe": ([vp, vp, u64, vp], ctypes.c_int),
        "ds_restore_begin": ([vp, vp, vp, P(vp)], ctypes.c_int),
        "ds_restore_next_slot": ([vp, P(vp), P(u64), P(u64)], ctypes.c_int),
        "ds_restore_submit": ([vp, vp], ctypes.c_int),
        "ds_flush_start": ([vp, ctypes.c_char_p, u32, u32, P(vp)], ctypes.c_int),
        "ds_flush_wait": ([vp, P(u64), P(ctypes.c_double)], ctypes.c_int),
        "ds_restore_from_file": ([vp, vp, ctypes.c_char_p, u32, u32, vp, P(vp)], ctypes.c_int),
        "ds_last_errno": ([], ctypes.c_int),
        "ds_plan_shard_shape": ([vp, sz, P(u32), P(ctypes.c_int64)], ctypes.c_int),
        "ds_ckpt_create": ([ctypes.c_char_p, vp, u32, P(vp)], ctypes.c_int),
        "ds_ckpt_flush_snapshot": ([vp, vp, u32], ctypes.c_int),
        "ds_ckpt_write_region": ([vp, u64, vp, u64], ctypes.c_int),
        "ds_ckpt_append": ([vp, u64, vp, u64], ctypes.c_int),
        "ds_ckpt_finish": ([vp, P(u64), P(ctypes.c_double)], ctypes.c_int),
        "ds_ckpt_open": ([ctypes.c_char_p, P(vp)], ctypes.c_int),
        "ds_ckpt_close": ([vp], ctypes.c_int),
        "ds_ckpt_layout_info": ([vp, P(ds_ckpt_layout)], ctypes.c_int),
        "ds_ckpt_tensor_info": ([vp, sz, P(ds_ckpt_tensor)], ctypes.c_int),
        "ds_ckpt_object_at": ([vp, sz, P(u64), P(u64)], ctypes.c_int),
        "ds_ckpt_object_read": ([vp, u64, vp, u64, P(u64)], ctypes.c_int),
        "ds_ckpt_matches_plan": ([vp, vp], ctypes.c_int),
        "ds_ckpt_restore": ([vp, vp, vp, u32, u32, vp, P(vp)], ctypes.c_int),
        "ds_event_trace": ([vp, P(ds_trace_rec), sz, P(sz)], ctypes.c_int),
        "ds_image_diff": ([vp, vp, u64, u64, vp, vp], ctypes.c_int),
        "ds_image_compress": ([vp, u64, u64, vp, vp, vp, vp, vp], ctypes.c_int),
        "ds_ckpt_append_from": ([vp, u64, ds_chunk_provider, vp, P(u64)], ctypes.c_int),
        "ds_plan_create_files": ([P(ds_shard_desc), P(u32), sz, u32, u64, u32, P(vp)], ctypes.c_int),
        "ds_layout_assign_files": ([P(ds_shard_desc), P(u32), sz, u32, u64, P(u64), P(u64)], ctypes.c_int),
        "ds_plan_file": ([vp, u32, P(u64), P(u64)], ctypes.c_int),
        "ds_plan_shard_file": ([vp, sz, P(u32), P(u64)], ctypes.c_int),
        "ds_flush_start_files": ([vp, P(ctypes.c_char_p), u32, u32, u32, P(vp)], ctypes.c_int),
        "ds_restore_from_files": ([vp, vp, P(ctypes.c_char_p), u32, u32, u32, vp, P(vp)], ctypes.c_int),
        "ds_ckpt_create_part": ([ctypes.c_char_p, vp, u32, u32, P(vp)], ctypes.c_int),
        "ds_ckpt_flush_snapshot_parts": ([P(vp), u32, vp, u32], ctypes.c_int),
        "ds_ckpt_matches_plan_part": ([vp, vp, u32], ctypes.c_int),
        "ds_ckpt_restore_parts": ([P(vp), u32, vp, vp, u32, u32, vp, P(vp)], ctypes.c_int),
    }
    for name, (args, res) in sig.items():
        fn = getattr(L, name)
        fn.argtypes = args
        fn.restype = res
    return L


_lib = _load()


def _check(rc: int, where: str) -> int:
    if rc < 0:
        raise DsError(rc, where)
    return rc


# ---- descriptor tables ------------------------------------------------------

def make_descs(shards: Sequence, base_address: int):
    """ctypes table from entries with .dtype (name or code) .shape .strides
    .byte_offset .tensor_id; `base_address` is the device address the byte
    offsets are relative to.  file_offset is left 0."""
    codes = {"f32": DS_F32, "bf16": DS_BF16, "f16": DS_F16, "i64": DS_I64, "u8": DS_U8}
    arr = (ds_shard_desc * max(len(shards), 1))()
    for i, s in enumerate(shards):
        d = arr[i]
        d.base = base_address + s.byte_offset
        d.dtype = codes[s.dtype] if isinstance(s.dtype, str) else int(s.dtype)
        d.ndim = len(s.shape)
        for j, (e, st) in enumerate(zip(s.shape, s.strides)):
            d.shape[j] = e
            d.strides[j] = st
        d.tensor_id = s.tensor_id
        d.file_offset = 0
    return arr


def make_descs_from_tensors(tensors: Sequence, tensor_ids: Optional[Sequence[int]] = None):
    """ctypes table straight from torch tensors on the GPU (any views: sliced,
    transposed, expanded dimensions excluded): device address, dtype, shape and
    element strides as torch reports them.  file_offset is left 0.  The caller
    keeps the tensors alive for as long as a plan made from the table is used."""
    import torch
    codes = {torch.float32: DS_F32, torch.bfloat16: DS_BF16, torch.float16: DS_F16, torch.int64: DS_I64,
             torch.uint8: DS_U8}
    arr = (ds_shard_desc * max(len(tensors), 1))()
    for i, t in enumerate(tensors):
        if t.dtype not in codes:
            raise TypeError(f"tensor {i}: dtype {t.dtype} has no ds_dtype")
        if not t.is_cuda:
            raise ValueError(f"tensor {i} is not in device memory")
        if t.dim() > DS_MAX_DIMS:
            raise ValueError(f"tensor {i} has more than {DS_MAX_DIMS} dimensions")
        d = arr[i]
        d.base = t.data_ptr()
        d.dtype = codes[t.dtype]
        d.ndim = t.dim()
        for j, (e, st) in enumerate(zip(t.shape, t.stride())):
            d.shape[j] = e
            d.strides[j] = st
        d.tensor_id = tensor_ids[i] if tensor_ids is not None else i
        d.file_offset = 0
    return arr


# ---- the entry points, same names as the C ABI -------------------------------

def ds_itemsize(dtype: int) -> int:
    return int(_lib.ds_itemsize(dtype))


def ds_layout_assign(descs, n: int, align: int) -> int:
    total = ctypes.c_uint64(0)
    _check(_lib.ds_layout_assign(descs, n, align, ctypes.byref(total)), "ds_layout_assign")
    return int(total.value)


def ds_plan_create(descs, n: int, align: int, flags: int = 0) -> int:
    out = ctypes.c_void_p(0)
    _check(_lib.ds_plan_create(descs, n, align, flags, ctypes.byref(out)), "ds_plan_create")
    return int(out.value)


def _u32_array(values: Sequence[int]):
    return (ctypes.c_uint32 * max(len(values), 1))(*values)


def _path_array(paths: Sequence[str]):
    return (ctypes.c_char_p * max(len(paths), 1))(*[p.encode() for p in paths])


def _handle_array(handles: Sequence[int]):
    return (ctypes.c_void_p * max(len(handles), 1))(*handles)


def ds_layout_assign_files(descs, file_of: Sequence[int], n: int, n_files: int, align: int) -> Tuple[List[int], int]:
    """(tensor-region length of every file, their sum = the image length)."""
    regions = (ctypes.c_uint64 * n_files)()
    total = ctypes.c_uint64(0)
    _check(_lib.ds_layout_assign_files(descs, _u32_array(file_of), n, n_files, align, regions, ctypes.byref(total)),
           "ds_layout_assign_files")
    return [int(r) for r in regions], int(total.value)


def ds_plan_create_files(descs, file_of: Sequence[int], n: int, n_files: int, align: int, flags: int = 0) -> int:
    out = ctypes.c_void_p(0)
    _check(_lib.ds_plan_create_files(descs, _u32_array(file_of), n, n_files, align, flags, ctypes.byref(out)),
           "ds_plan_create_files")
    return int(out.value)


def ds_plan_file(plan: int, f: int) -> Tuple[int, int]:
    """(where file f's tensor region starts in the image, its length)."""
    begin, nbytes = ctypes.c_uint64(0), ctypes.c_uint64(0)
    _check(_lib.ds_plan_file(plan, f, ctypes.byref(begin), ctypes.byref(nbytes)), "ds_plan_file")
    return int(begin.value), int(nbytes.value)


def ds_plan_shard_file(plan: int, i: int) -> Tuple[int, int]:
    """(file of manifest entry i, its offset in the image)."""
    f, off = ctypes.c_uint32(0), ctypes.c_uint64(0)
    _check(_lib.ds_plan_shard_file(plan, i, ctypes.byref(f), ctypes.byref(off)), "ds_plan_shard_file")
    return int(f.value), int(off.value)


def ds_plan_destroy(plan: int) -> None:
    _check(_lib.ds_plan_destroy(plan), "ds_plan_destroy")


def ds_plan_info(plan: int) -> dict:
    st = ds_plan_stats()
    _check(_lib.ds_plan_info(plan, ctypes.byref(st)), "ds_plan_info")
    return {n: int(getattr(st, n)) for n, _ in ds_plan_stats._fields_}


def ds_plan_shard(plan: int, i: int) -> Tuple[int, int, int, int]:
    tid, dt, off, nb = ctypes.c_uint64(), ctypes.c_uint32(), ctypes.c_uint64(), ctypes.c_uint64()
    _check(_lib.ds_plan_shard(plan, i, ctypes.byref(tid), ctypes.byref(dt), ctypes.byref(off), ctypes.byref(nb)),
           "ds_plan_shard")
    return int(tid.value), int(dt.value), int(off.value), int(nb.value)


def ds_pack(plan: int, dst_dev: int, img_lo: int, img_hi: int, stream: int = 0) -> None:
    _check(_lib.ds_pack(plan, dst_dev, img_lo, img_hi, stream), "ds_pack")


def ds_pack_noalloc(plan: int, dst_dev: int, img_lo: int, img_hi: int, stream: int = 0) -> None:
    _check(_lib.ds_pack_noalloc(plan, dst_dev, img_lo, img_hi, stream), "ds_pack_noalloc")


def ds_unpack(plan: int, src_dev: int, img_lo: int, img_hi: int, stream: int = 0) -> None:
    _check(_lib.ds_unpack(plan, src_dev, img_lo, img_hi, stream), "ds_unpack")


def ds_engine_create(host_ring_bytes: int = 0, d2h_chunk_bytes: int = 0, stage_slot_bytes: int = 0,
                     stage_slots: int = 0, pack_grid_limit: int = 0, flags: int = 0, copy_streams: int = 0,
                     first_launch_bytes: int = 0) -> int:
    opts = ds_engine_opts(host_ring_bytes, d2h_chunk_bytes, stage_slot_bytes, stage_slots, pack_grid_limit, flags,
                          copy_streams, first_launch_bytes)
    out = ctypes.c_void_p(0)
    _check(_lib.ds_engine_create(ctypes.byref(opts), ctypes.byref(out)), "ds_engine_create")
    return int(out.value)


def ds_engine_destroy(engine: int) -> None:
    _check(_lib.ds_engine_destroy(engine), "ds_engine_destroy")


def ds_snapshot_async(engine: int, plan: int, compute_stream: int = 0) -> int:
    out = ctypes.c_void_p(0)
    _check(_lib.ds_snapshot_async(engine, plan, compute_stream, ctypes.byref(out)), "ds_snapshot_async")
    return int(out.value)


def ds_event_wait_on_stream(ev: int, stream: int = 0) -> None:
    _check(_lib.ds_event_wait_on_stream(ev, stream), "ds_event_wait_on_stream")


def ds_event_wait_captured(ev: int) -> None:
    _check(_lib.ds_event_wait_captured(ev), "ds_event_wait_captured")


def ds_event_query(ev: int) -> int:
    return _check(_lib.ds_event_query(ev), "ds_event_query")


def ds_event_wait(ev: int) -> None:
    _check(_lib.ds_event_wait(ev), "ds_event_wait")


def ds_snapshot_next_chunk(ev: int) -> Optional[Tuple[int, int, int]]:
    """(host address, file offset, length) of the next chunk, or None at the end."""
    ptr, off, ln = ctypes.c_void_p(0), ctypes.c_uint64(0), ctypes.c_uint64(0)
    rc = _check(_lib.ds_snapshot_next_chunk(ev, ctypes.byref(ptr), ctypes.byref(off), ctypes.byref(ln)),
                "ds_snapshot_next_chunk")
    if rc == DS_EOF:
        return None
    return int(ptr.value), int(off.value), int(ln.value)


def ds_snapshot_release_chunk(ev: int, host_ptr: int) -> None:
    _check(_lib.ds_snapshot_release_chunk(ev, host_ptr), "ds_snapshot_release_chunk")


def ds_event_stats(ev: int) -> dict:
    st = ds_snapshot_stats()
    _check(_lib.ds_event_stats(ev, ctypes.byref(st)), "ds_event_stats")
    return {n: getattr(st, n) for n, _ in ds_snapshot_stats._fields_}


def ds_event_destroy(ev: int) -> None:
    _check(_lib.ds_event_destroy(ev), "ds_event_destroy")


def ds_strerror(code: int) -> str:
    return _lib.ds_strerror(code).decode()


def ds_last_hip_error() -> int:
    return int(_lib.ds_last_hip_error())


def ds_config_set(key: str, value: int) -> None:
    _check(_lib.ds_config_set(key.encode(), value), f"ds_config_set({key})")


def ds_config_get(key: str) -> int:
    v = ctypes.c_uint64(0)
    _check(_lib.ds_config_get(key.encode(), ctypes.byref(v)), f"ds_config_get({key})")
    return int(v.value)


def ds_copy_probe(dst_dev: int, src_dev: int, nbytes: int, stream: int = 0) -> None:
    _check(_lib.ds_copy_probe(dst_dev, src_dev, nbytes, stream), "ds_copy_probe")


def ds_restore_begin(engine: int, plan: int, compute_stream: int = 0) -> int:
    out = ctypes.c_void_p(0)
    _check(_lib.ds_restore_begin(engine, plan, compute_stream, ctypes.byref(out)), "ds_restore_begin")
    return int(out.value)


def ds_restore_next_slot(ev: int) -> Optional[Tuple[int, int, int]]:
    """(host address, file offset, length) of the next ring slot to fill, or None at the end."""
    ptr, off, ln = ctypes.c_void_p(0), ctypes.c_uint64(0), ctypes.c_uint64(0)
    rc = _check(_lib.ds_restore_next_slot(ev, ctypes.byref(ptr), ctypes.byref(off), ctypes.byref(ln)),
                "ds_restore_next_slot")
    if rc == DS_EOF:
        return None
    return int(ptr.value), int(off.value), int(ln.value)


def ds_restore_submit(ev: int, host_ptr: int) -> None:
    _check(_lib.ds_restore_submit(ev, host_ptr), "ds_restore_submit")


def ds_flush_start(ev: int, path: str, threads: int = 0, flags: int = 0) -> int:
    out = ctypes.c_void_p(0)
    _check(_lib.ds_flush_start(ev, path.encode(), threads, flags, ctypes.byref(out)), "ds_flush_start")
    return int(out.value)


def ds_flush_start_files(ev: int, paths: Sequence[str], threads: int = 0, flags: int = 0) -> int:
    out = ctypes.c_void_p(0)
    _check(_lib.ds_flush_start_files(ev, _path_array(paths), len(paths), threads, flags, ctypes.byref(out)),
           "ds_flush_start_files")
    return int(out.value)


def ds_flush_wait(flush: int) -> Tuple[int, float]:
    """(bytes written, seconds from ds_flush_start to the last write)."""
    nbytes, secs = ctypes.c_uint64(0), ctypes.c_double(0)
    _check(_lib.ds_flush_wait(flush, ctypes.byref(nbytes), ctypes.byref(secs)), "ds_flush_wait")
    return int(nbytes.value), float(secs.value)


def ds_restore_from_file(engine: int, plan: int, path: str, threads: int = 0, flags: int = 0,
                         compute_stream: int = 0) -> int:
    out = ctypes.c_void_p(0)
    _check(_lib.ds_restore_from_file(engine, plan, path.encode(), threads, flags, compute_stream,
                                     ctypes.byref(out)), "ds_restore_from_file")
    return int(out.value)


def ds_restore_from_files(engine: int, plan: int, paths: Sequence[str], threads: int = 0, flags: int = 0,
                          compute_stream: int = 0) -> int:
    out = ctypes.c_void_p(0)
    _check(_lib.ds_restore_from_files(engine, plan, _path_array(paths), len(paths), threads, flags, compute_stream,
                                      ctypes.byref(out)), "ds_restore_from_files")
    return int(out.value)


def ds_last_errno() -> int:
    return int(_lib.ds_last_errno())


def ds_plan_shard_shape(plan: int, i: int) -> Tuple[int, ...]:
    nd = ctypes.c_uint32(0)
    shape = (ctypes.c_int64 * DS_MAX_DIMS)()
    _check(_lib.ds_plan_shard_shape(plan, i, ctypes.byref(nd), shape), "ds_plan_shard_shape")
    return tuple(int(shape[j]) for j in range(nd.value))


def ds_ckpt_create(path: str, plan: int, flags: int = 0) -> int:
    out = ctypes.c_void_p(0)
    _check(_lib.ds_ckpt_create(path.encode(), plan, flags, ctypes.byref(out)), "ds_ckpt_create")
    return int(out.value)


def ds_ckpt_create_part(path: str, plan: int, file: int, flags: int = 0) -> int:
    out = ctypes.c_void_p(0)
    _check(_lib.ds_ckpt_create_part(path.encode(), plan, file, flags, ctypes.byref(out)), "ds_ckpt_create_part")
    return int(out.value)


def ds_ckpt_flush_snapshot_parts(parts: Sequence[int], snapshot: int, threads: int = 0) -> None:
    _check(_lib.ds_ckpt_flush_snapshot_parts(_handle_array(parts), len(parts), snapshot, threads),
           "ds_ckpt_flush_snapshot_parts")


def ds_ckpt_flush_snapshot(ckpt: int, snapshot: int, threads: int = 0) -> None:
    _check(_lib.ds_ckpt_flush_snapshot(ckpt, snapshot, threads), "ds_ckpt_flush_snapshot")


def ds_ckpt_write_region(ckpt: int, file_off: int, host_ptr: int, nbytes: int) -> None:
    _check(_lib.ds_ckpt_write_region(ckpt, file_off, host_ptr, nbytes), "ds_ckpt_write_region")


def ds_ckpt_append(ckpt: int, object_id: int, data: bytes) -> None:
    _check(_lib.ds_ckpt_append(ckpt, object_id, ctypes.c_char_p(data) if data else None, len(data)),
           "ds_ckpt_append")


def ds_ckpt_append_from(ckpt: int, object_id: int, chunks) -> int:
    """Drains an iterable of bytes-like chunks (an object state provider) into the log; returns the number of
    chunks appended.  The iterable is pulled from inside the library, one chunk at a time."""
    it = iter(chunks)
    keep = []                                            # the chunk handed out last stays alive until the next call

    def next_chunk(_ctx, data, length):
        try:
            b = bytes(next(it))
        except StopIteration:
            return 0
        except Exception:                                # noqa: BLE001 -- reported as the provider's error
            return DS_EINVAL
        keep[:] = [ctypes.create_string_buffer(b, len(b)) if b else None]
        data[0] = ctypes.cast(keep[0], ctypes.c_void_p).value if b else None
        length[0] = len(b)
        return 1
    n = ctypes.c_uint64(0)
    _check(_lib.ds_ckpt_append_from(ckpt, object_id, ds_chunk_provider(next_chunk), None, ctypes.byref(n)),
           "ds_ckpt_append_from")
    return int(n.value)


def ds_ckpt_finish(ckpt: int) -> Tuple[int, float]:
    """(file length, seconds since ds_ckpt_create)."""
    nbytes, secs = ctypes.c_uint64(0), ctypes.c_double(0)
    _check(_lib.ds_ckpt_finish(ckpt, ctypes.byref(nbytes), ctypes.byref(secs)), "ds_ckpt_finish")
    return int(nbytes.value), float(secs.value)


def ds_ckpt_open(path: str) -> int:
    out = ctypes.c_void_p(0)
    _check(_lib.ds_ckpt_open(path.encode(), ctypes.byref(out)), "ds_ckpt_open")
    return int(out.value)


def ds_ckpt_close(reader: int) -> None:
    _check(_lib.ds_ckpt_close(reader), "ds_ckpt_close")


def ds_ckpt_layout_info(reader: int) -> dict:
    lay = ds_ckpt_layout()
    _check(_lib.ds_ckpt_layout_info(reader, ctypes.byref(lay)), "ds_ckpt_layout_info")
    return {n: int(getattr(lay, n)) for n, _ in ds_ckpt_layout._fields_}


def ds_ckpt_tensor_info(reader: int, i: int) -> dict:
    t = ds_ckpt_tensor()
    _check(_lib.ds_ckpt_tensor_info(reader, i, ctypes.byref(t)), "ds_ckpt_tensor_info")
    return {"tensor_id": int(t.tensor_id), "dtype": int(t.dtype), "shape": tuple(int(t.shape[j]) for j in range(t.ndim)),
            "file_offset": int(t.file_offset), "nbytes": int(t.nbytes)}


def ds_ckpt_object_at(reader: int, k: int) -> Tuple[int, int]:
    oid, nb = ctypes.c_uint64(0), ctypes.c_uint64(0)
    _check(_lib.ds_ckpt_object_at(reader, k, ctypes.byref(oid), ctypes.byref(nb)), "ds_ckpt_object_at")
    return int(oid.value), int(nb.value)


def ds_ckpt_object_read(reader: int, object_id: int) -> bytes:
    ln = ctypes.c_uint64(0)
    rc = _lib.ds_ckpt_object_read(reader, object_id, None, 0, ctypes.byref(ln))
    if rc not in (DS_OK, DS_ERANGE):
        _check(rc, "ds_ckpt_object_read")
    buf = ctypes.create_string_buffer(max(int(ln.value), 1))
    _check(_lib.ds_ckpt_object_read(reader, object_id, buf, ln.value, ctypes.byref(ln)), "ds_ckpt_object_read")
    return buf.raw[:ln.value]


def ds_ckpt_matches_plan(reader: int, plan: int) -> None:
    _check(_lib.ds_ckpt_matches_plan(reader, plan), "ds_ckpt_matches_plan")


def ds_ckpt_matches_plan_part(reader: int, plan: int, file: int) -> None:
    _check(_lib.ds_ckpt_matches_plan_part(reader, plan, file), "ds_ckpt_matches_plan_part")


def ds_ckpt_restore_parts(readers: Sequence[int], engine: int, plan: int, threads: int = 0, flags: int = 0,
                          compute_stream: int = 0) -> int:
    out = ctypes.c_void_p(0)
    _check(_lib.ds_ckpt_restore_parts(_handle_array(readers), len(readers), engine, plan, threads, flags,
                                      compute_stream, ctypes.byref(out)), "ds_ckpt_restore_parts")
    return int(out.value)


def ds_ckpt_restore(reader: int, engine: int, plan: int, threads: int = 0, flags: int = 0,
                    compute_stream: int = 0) -> int:
    out = ctypes.c_void_p(0)
    _check(_lib.ds_ckpt_restore(reader, engine, plan, threads, flags, compute_stream, ctypes.byref(out)),
           "ds_ckpt_restore")
    return int(out.value)


def ds_event_trace(ev: int) -> List[dict]:
    """Records of a finished snapshot: gather launches (kind 0), then, on a tracing engine, the chunk copies
    (kind 1); times in milliseconds since the request."""
    n = ctypes.c_size_t(0)
    _check(_lib.ds_event_trace(ev, None, 0, ctypes.byref(n)), "ds_event_trace")
    recs = (ds_trace_rec * max(n.value, 1))()
    _check(_lib.ds_event_trace(ev, recs, n.value, ctypes.byref(n)), "ds_event_trace")
    return [{f: getattr(recs[i], f) for f, _ in ds_trace_rec._fields_} for i in range(n.value)]


def ds_image_diff(image_a_dev: int, image_b_dev: int, nbytes: int, block_bytes: int, changed_dev: int,
                  stream: int = 0) -> None:
    _check(_lib.ds_image_diff(image_a_dev, image_b_dev, nbytes, block_bytes, changed_dev, stream), "ds_image_diff")


def ds_image_compress(image_dev: int, nbytes: int, block_bytes: int, keep_dev: int, pos_dev: int, patterns_dev: int,
                      packed_dev: int, stream: int = 0) -> None:
    _check(_lib.ds_image_compress(image_dev, nbytes, block_bytes, keep_dev, pos_dev, patterns_dev, packed_dev, stream),
           "ds_image_compress")
