"""CPU-only tests of the library's host side: the shared object loads and
exports every declared symbol; layout and plan validation (no device calls:
plans are created with DS_PLAN_HOST_ONLY)."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2601_16956_amd as ds
import workloads as W
from oracle import ds_oracle as orc
from workloads.configs import Shard

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "datastates.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(ds_[a-z0-9_]+)\s*\(", header))
    assert declared == set(ds.EXPORTS), declared ^ set(ds.EXPORTS)
    L = ctypes.CDLL(ds.LIB_PATH)
    for name in declared:
        assert getattr(L, name) is not None


def test_struct_sizes_match_the_header():
    assert ctypes.sizeof(ds.ds_shard_desc) == 8 + 4 + 4 + 48 + 48 + 8 + 8
    assert ctypes.sizeof(ds.ds_engine_opts) == 48
    assert ctypes.sizeof(ds.ds_plan_stats) == 80


def test_strerror_covers_all_codes():
    for code in (0, 1, 2, -1, -2, -3, -4, -5, -6, -7, -8, -9, -10, -11):
        assert "unknown" not in ds.ds_strerror(code)
    assert "unknown" in ds.ds_strerror(-99)


def _descs(shards, base=0x10000):
    return ds.make_descs(shards, base)


@pytest.mark.parametrize("maker", [
    lambda: W.tiny_gpt(),
    lambda: W.fragmentation(2000, max_bytes=1 << 16, seed=8),
    lambda: W.llama_rank("mini", 128, 352, 4, 2, 512, 2, 4, 8, seed=5, workers=1),
])
def test_layout_assign_agrees_with_oracle_layout(maker):
    w = maker()
    n = len(w.shards)
    d = _descs(w.shards)
    total = ds.ds_layout_assign(d, n, w.align)
    tab = orc.table(w.shards, w.arena.ctypes.data)
    assert total == orc.layout(tab, n, w.align)
    assert [int(d[i].file_offset) for i in range(n)] == [int(tab[i].file_offset) for i in range(n)]
    plan = ds.ds_plan_create(d, n, w.align, ds.DS_PLAN_HOST_ONLY | ds.DS_PLAN_STRICT)
    info = ds.ds_plan_info(plan)
    assert info["total_bytes"] == total and info["payload_bytes"] == w.payload_bytes
    assert info["n_shards"] == n and info["align"] == w.align
    assert info["n_chunks"] == -(-total // info["chunk_bytes"])
    for i, s in enumerate(w.shards):
        tid, dt, off, nb = ds.ds_plan_shard(plan, i)
        assert (tid, off, nb) == (s.tensor_id, int(d[i].file_offset), s.nbytes)
    ds.ds_plan_destroy(plan)


def _plan_rc(shards, align, offsets=None, flags=0, base=0x10000):
    d = _descs(shards, base)
    n = len(shards)
    try:
        if offsets is None:
            ds.ds_layout_assign(d, n, align)
        else:
            for i, off in enumerate(offsets):
                d[i].file_offset = off
        plan = ds.ds_plan_create(d, n, align, flags | ds.DS_PLAN_HOST_ONLY)
    except ds.DsError as e:
        return e.code
    ds.ds_plan_destroy(plan)
    return 0


def test_plan_validation_codes():
    ok = [Shard("a", "f32", (4, 4), (4, 1), 0, 0), Shard("b", "u8", (100,), (1,), 256, 1)]
    assert _plan_rc(ok, 64) == 0
    assert _plan_rc(ok, 48) == ds.DS_EINVAL                       # not a power of two
    assert _plan_rc(ok, 8) == ds.DS_EINVAL                        # below 16
    assert _plan_rc(ok, 64, offsets=[0, 32]) == ds.DS_EALIGN
    assert _plan_rc(ok, 64, offsets=[0, 0]) == ds.DS_EOVERLAP
    assert _plan_rc(ok, 16, offsets=[0, 48]) == ds.DS_EOVERLAP    # a is 64 bytes
    assert _plan_rc(ok, 64, offsets=[0, 128], flags=ds.DS_PLAN_STRICT) == ds.DS_EGAP
    assert _plan_rc(ok, 64, offsets=[0, 128]) == 0                # holes allowed unless strict
    assert _plan_rc(ok, 64, offsets=[64, 128], flags=ds.DS_PLAN_STRICT) == ds.DS_EGAP   # hole at the start
    assert _plan_rc(ok, 64, offsets=[128, 0]) == 0                # any order
    bad_dtype = [Shard("x", 7, (4,), (1,), 0, 0)]
    assert _plan_rc(bad_dtype, 64) == ds.DS_EINVAL
    assert _plan_rc([Shard("x", "f32", (4, -1), (1, 1), 0, 0)], 64, offsets=[0]) == ds.DS_EINVAL
    assert _plan_rc([Shard("x", "f32", (4, 4), (0, 1), 0, 0)], 64) == ds.DS_EINVAL      # zero stride
    assert _plan_rc([Shard("x", "f32", (4, 4), (-4, 1), 0, 0)], 64) == ds.DS_EINVAL     # negative stride
    assert _plan_rc([Shard("x", "f32", (4, 4), (3, 1), 0, 0)], 64) == ds.DS_EOVERLAP    # rows overlap
    assert _plan_rc([Shard("x", "f32", (4, 4), (1, 1), 0, 0)], 64) == ds.DS_EOVERLAP
    assert _plan_rc([Shard("x", "f32", (4, 4), (1, 4), 0, 0)], 64) == 0                 # transposed is fine
    # strides that do not nest are decided by writing the addresses out: (3,2)/(2,3) -> 0,3,2,5,4,7 is a view,
    # (3,2)/(2,2) -> 0,2,2,4,4,6 is not; against a brute-force set for every small stride pair
    assert _plan_rc([Shard("x", "f32", (3, 2), (2, 3), 0, 0)], 64) == 0
    assert _plan_rc([Shard("x", "f32", (3, 2), (2, 2), 0, 0)], 64) == ds.DS_EOVERLAP
    for s0 in range(1, 9):
        for s1 in range(1, 9):
            for s2 in (1, 5):
                at = [i * s0 + j * s1 + k * s2 for i in range(3) for j in range(4) for k in range(2)]
                want = 0 if len(set(at)) == len(at) else ds.DS_EOVERLAP
                assert _plan_rc([Shard("x", "bf16", (3, 4, 2), (s0, s1, s2), 0, 0)], 64) == want, (s0, s1, s2)
    # beyond 2^20 elements a view whose strides do not nest is refused
    # (even addresses, then odd ones from 3 on: no address twice, yet 3 lies inside the reach of the stride 2)
    assert _plan_rc([Shard("x", "u8", (1 << 19, 2), (2, 3), 0, 0)], 64) == 0
    assert _plan_rc([Shard("x", "u8", (1 << 20, 2), (2, 3), 0, 0)], 64) == ds.DS_EOVERLAP
    assert _plan_rc([Shard("x", "f32", (1, 4), (0, 1), 0, 0)], 64) == 0                 # stride of an extent 1 is free
    assert _plan_rc([Shard("x", "f32", (4,), (1,), 2, 0)], 64) == ds.DS_EINVAL          # base not element-aligned
    assert _plan_rc([Shard("x", "f32", (4,), (1,), 0, 0)], 64, base=0) == ds.DS_EINVAL  # null base
    assert _plan_rc([Shard("x", "f32", (0,), (1,), 0, 0)], 64, base=0) == 0             # ... unless empty
    assert _plan_rc([], 64) == 0


def test_seven_dims_rejected():
    d = (ds.ds_shard_desc * 1)()
    d[0].base = 0x1000
    d[0].dtype = ds.DS_U8
    d[0].ndim = 7
    out = ctypes.c_void_p()
    assert ds._lib.ds_plan_create(d, 1, 64, ds.DS_PLAN_HOST_ONLY, ctypes.byref(out)) == ds.DS_EINVAL
    assert out.value is None                                      # untouched on failure


def test_unknown_flags_and_memory_check_on_a_host_only_plan_are_rejected():
    d = _descs([Shard("a", "u8", (64,), (1,), 0, 0)])
    ds.ds_layout_assign(d, 1, 64)
    out = ctypes.c_void_p()
    for flags in (8, 0x100, ds.DS_PLAN_HOST_ONLY | ds.DS_PLAN_CHECK_MEMORY):
        assert ds._lib.ds_plan_create(d, 1, 64, flags, ctypes.byref(out)) == ds.DS_EINVAL
        assert out.value is None
    assert "allocation" in ds.ds_strerror(ds.DS_EFAULT)


def test_host_only_plan_cannot_be_packed():
    d = _descs([Shard("a", "u8", (64,), (1,), 0, 0)])
    ds.ds_layout_assign(d, 1, 64)
    plan = ds.ds_plan_create(d, 1, 64, ds.DS_PLAN_HOST_ONLY)
    with pytest.raises(ds.DsError) as e:
        ds.ds_pack(plan, 0x1000, 0, 64, 0)
    assert e.value.code == ds.DS_EINVAL
    ds.ds_plan_destroy(plan)


def test_config_keys():
    assert ds.ds_config_get("chunk_bytes") == 16 << 10
    for bad in (1000, 4096, 64 << 10, 128 << 10):
        with pytest.raises(ds.DsError):
            ds.ds_config_set("chunk_bytes", bad)
    with pytest.raises(ds.DsError):
        ds.ds_config_set("no_such_key", 1)
    with pytest.raises(ds.DsError):
        ds.ds_config_set("variant", 6)
    assert ds.ds_config_get("grid_limit") == 0
    ds.ds_config_set("grid_limit", 64)
    assert ds.ds_config_get("grid_limit") == 64
    ds.ds_config_set("grid_limit", 0)
    with pytest.raises(ds.DsError):
        ds.ds_config_set("grid_limit", 1 << 31)
    assert ds.ds_config_get("io_uring_available") in (0, 1)
    with pytest.raises(ds.DsError):
        ds.ds_config_set("io_uring_available", 1)
    ds.ds_config_set("chunk_bytes", 32 << 10)
    d = _descs([Shard("a", "u8", (1 << 20,), (1,), 0, 0)])
    ds.ds_layout_assign(d, 1, 64)
    plan = ds.ds_plan_create(d, 1, 64, ds.DS_PLAN_HOST_ONLY)
    assert ds.ds_plan_info(plan)["n_chunks"] == 32
    ds.ds_plan_destroy(plan)
    ds.ds_config_set("chunk_bytes", 16 << 10)


def test_plain_c_program_uses_the_header_and_the_library(tmp_path):
    """The header is C: a C99 program built with gcc against it and the shared
    library reports the struct layouts (compared with the binding's ctypes
    mirrors) and runs layout, a host-only plan and a checkpoint file."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc here")
    exe = str(tmp_path / "abi_check")
    libdir = os.path.dirname(ds.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "c_abi", "abi_check.c"), "-o", exe,
                    "-L", libdir, "-ldatastates_hip", "-Wl,-rpath," + libdir,
                    "-Wl,--allow-shlib-undefined"], check=True)
    hip_dirs = [os.path.dirname(p) for p in ds.hip_runtime_in_use()] + ["/opt/rocm/lib"]
    env = dict(os.environ, LD_LIBRARY_PATH=":".join(hip_dirs + [os.environ.get("LD_LIBRARY_PATH", "")]))
    ckpt = str(tmp_path / "c.ckpt")
    out = subprocess.run([exe, ckpt], check=True, capture_output=True, text=True, env=env).stdout
    facts = dict(line.rsplit(" ", 1) for line in out.splitlines() if line.startswith(("sizeof", "offsetof")))
    assert int(facts["sizeof ds_shard_desc"]) == ctypes.sizeof(ds.ds_shard_desc)
    for f in ("shape", "strides", "tensor_id", "file_offset"):
        assert int(facts[f"offsetof ds_shard_desc.{f}"]) == getattr(ds.ds_shard_desc, f).offset
    assert int(facts["sizeof ds_plan_stats"]) == ctypes.sizeof(ds.ds_plan_stats)
    assert int(facts["sizeof ds_engine_opts"]) == ctypes.sizeof(ds.ds_engine_opts)
    assert int(facts["offsetof ds_engine_opts.first_launch_bytes"]) == ds.ds_engine_opts.first_launch_bytes.offset
    assert int(facts["sizeof ds_snapshot_stats"]) == ctypes.sizeof(ds.ds_snapshot_stats)
    assert int(facts["sizeof ds_ckpt_layout"]) == ctypes.sizeof(ds.ds_ckpt_layout)
    assert int(facts["sizeof ds_ckpt_tensor"]) == ctypes.sizeof(ds.ds_ckpt_tensor)
    assert int(facts["offsetof ds_ckpt_tensor.file_offset"]) == ds.ds_ckpt_tensor.file_offset.offset
    assert "total 3328 offsets 0 512 3072" in out                 # 400 B, 2400 B, 4 B at multiples of 256
    assert "payload 2804 shards 3 strided 1" in out
    assert "tensors 3 objects 2 chunks 3 object42 'hello world' tensor1 id 12 ndim 2 shape 30 20" in out
    # the file the C program wrote, read by the oracle's parser
    from oracle import ckpt_format as fmt
    back = fmt.parse_file(open(ckpt, "rb").read())
    assert back["objects"] == {7: b"x", 42: b"hello world"}
    assert [t[0] for t in back["tensors"]] == [11, 12, 13] and back["tensor_bytes"] == 3328
    floats = np.frombuffer(back["image"], dtype=np.float32)
    assert floats[0:100].tolist() == [float(i) for i in range(100)]
    assert floats[128 + 20 * 3: 128 + 20 * 3 + 3].tolist() == [7 + 48 * 3, 8 + 48 * 3, 9 + 48 * 3]
    assert floats[3072 // 4] == 5.0
    assert len(open(ckpt, "rb").read()) == 3328 + 24 + 3 * 80 + 3 * 32 + 64


def test_splice_of_the_kernels_on_the_host(tmp_path):
    """csrc/ds_splice.h, the routine every unit cut by the end of a run goes through in the kernels, compiled
    unchanged for the host: bytes [s, s+16) of a || b for every s, against plain slicing of the 32 bytes; and
    the byte-align primitive against its definition on the eight bytes lo || hi."""
    import shutil
    import subprocess
    if shutil.which("g++") is None:
        pytest.skip("no g++ here")
    so = str(tmp_path / "splice_host.so")
    subprocess.run(["g++", "-O2", "-Wall", "-Werror", "-fPIC", "-shared", "-I",
                    os.path.join(ROOT, "paper_2601_16956_amd", "csrc"),
                    os.path.join(ROOT, "tests", "c_abi", "splice_host.cpp"), "-o", so], check=True)
    lib = ctypes.CDLL(so)
    lib.align_bytes_host.restype = ctypes.c_uint32
    lib.align_bytes_host.argtypes = [ctypes.c_uint32] * 3
    rng = np.random.default_rng(7)
    patterns = [bytes(range(32)), bytes(range(255, 223, -1)), b"\xff" * 32, b"\x00" * 16 + b"\xff" * 16,
                b"\x80" * 32] + [rng.integers(0, 256, 32, dtype=np.uint8).tobytes() for _ in range(200)]
    out = (ctypes.c_ubyte * 16)()
    for both in patterns:
        a = (ctypes.c_ubyte * 16).from_buffer_copy(both[:16])
        b = (ctypes.c_ubyte * 16).from_buffer_copy(both[16:])
        for s in range(16):
            lib.splice_host(a, b, s, out)
            assert bytes(out) == both[s:s + 16], (both.hex(), s, bytes(out).hex())
        lo, hi = int.from_bytes(both[0:4], "little"), int.from_bytes(both[4:8], "little")
        for r in range(4):
            assert lib.align_bytes_host(hi, lo, r) == int.from_bytes(both[r:r + 4], "little")
