"""GPU parity: the HIP gather/scatter (through the C ABI) against the CPU
oracle, byte for byte, on the same seeded inputs.  Integer/byte work: the bar
is bit-exact (memcmp), never a float comparison -- the fragmentation inputs
contain NaN bit patterns."""
import numpy as np
import pytest

import workloads as W
from workloads.configs import Shard, Workload

pytestmark = pytest.mark.gpu


def _mods():
    import paper_2601_16956_amd as ds
    from oracle import ds_oracle as orc
    import gpu_util
    return ds, orc, gpu_util


SMALL = {
    "tiny_gpt": lambda: W.tiny_gpt(),
    "frag_small": lambda: W.fragmentation(3000, max_bytes=1 << 18, seed=101),
    "frag_tiny_only": lambda: W.fragmentation(5000, max_bytes=2048, seed=102),
    "frag_all_strided": lambda: W.fragmentation(800, max_bytes=1 << 19, strided_fraction=1.0, seed=103),
    "llama_mini": lambda: W.llama_rank("mini", 256, 704, 4, 2, 1024, 2, 4, 8, seed=5, workers=4),
    "frag_align16": lambda: W.fragmentation(2000, max_bytes=1 << 14, align=16, seed=104),
}


@pytest.mark.parametrize("name", list(SMALL))
def test_pack_matches_oracle(name):
    ds, orc, gu = _mods()
    w = SMALL[name]()
    print(f"[case] pack {name} shards={len(w.shards)} payload={w.payload_bytes}", flush=True)
    want, offs, _ = gu.oracle_image(w)
    dw = gu.DeviceWorkload(w)
    try:
        assert dw.offsets == offs and dw.total == want.size
        assert dw.info["payload_bytes"] == w.payload_bytes
        got = dw.pack()
        assert gu.first_mismatch(got, want) is None, gu.first_mismatch(got, want)
    finally:
        dw.close()


@pytest.mark.parametrize("name", list(SMALL))
def test_unpack_matches_oracle(name):
    """Restore into an arena of 0xA5: addressed elements get the image's bytes,
    every other byte keeps 0xA5 -- compared over the WHOLE arena."""
    ds, orc, gu = _mods()
    w = SMALL[name]()
    print(f"[case] unpack {name}", flush=True)
    img, offs, tab = gu.oracle_image(w)
    dw = gu.DeviceWorkload(w, arena_fill=0xA5)
    try:
        dw.unpack(img)
        got = dw.arena_host()
        w.arena[:] = 0xA5
        orc.unpack(tab, len(w.shards), img)
        assert gu.first_mismatch(got, w.arena) is None, gu.first_mismatch(got, w.arena)
    finally:
        dw.close()


@pytest.mark.parametrize("chunk_bytes", [8192, 16384, 32768])
@pytest.mark.parametrize("variant", [0, 1, 2, 3, 4, 5])
def test_chunk_sizes_and_kernel_variants(chunk_bytes, variant):
    ds, orc, gu = _mods()
    w = W.fragmentation(1500, max_bytes=1 << 19, seed=77)
    print(f"[case] chunk={chunk_bytes} variant={variant}", flush=True)
    want, offs, tab = gu.oracle_image(w)
    old_c, old_v = ds.ds_config_get("chunk_bytes"), ds.ds_config_get("variant")
    ds.ds_config_set("chunk_bytes", chunk_bytes)
    ds.ds_config_set("variant", variant)
    try:
        dw = gu.DeviceWorkload(w)
        assert dw.info["chunk_bytes"] == chunk_bytes
        got = dw.pack()
        assert gu.first_mismatch(got, want) is None, gu.first_mismatch(got, want)
        dw.arena.fill_(0xA5)
        dw.unpack(want)
        back = dw.arena_host()
        w.arena[:] = 0xA5
        orc.unpack(tab, len(w.shards), want)
        assert gu.first_mismatch(back, w.arena) is None
        dw.close()
    finally:
        ds.ds_config_set("chunk_bytes", old_c)
        ds.ds_config_set("variant", old_v)


@pytest.mark.parametrize("grid_limit", [1, 7, 8, 100, 4096])
def test_fewer_work_groups_than_chunks(grid_limit):
    """A launch limited to a few work-groups walks the interleaved rows of general
    and lean chunks in strides; every chunk must still be moved exactly once,
    and a gather straight into pinned HOST memory gives the same bytes."""
    ds, orc, gu = _mods()
    import torch
    w = W.fragmentation(700, max_bytes=1 << 18, seed=79)
    print(f"[case] grid_limit={grid_limit}", flush=True)
    want, offs, tab = gu.oracle_image(w)
    ds.ds_config_set("grid_limit", grid_limit)
    try:
        assert ds.ds_config_get("grid_limit") == grid_limit
        dw = gu.DeviceWorkload(w)
        got = dw.pack()
        assert gu.first_mismatch(got, want) is None, gu.first_mismatch(got, want)
        lo, hi = 16 * 1001, dw.total - 16 * 77                 # a cut range as well
        assert gu.first_mismatch(dw.pack(lo, hi), want[lo:hi]) is None
        host = torch.full((dw.total,), 0xFF, dtype=torch.uint8, pin_memory=True)
        ds.ds_pack(dw.plan, host.data_ptr(), 0, dw.total, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert gu.first_mismatch(host.numpy(), want) is None
        dw.arena.fill_(0xA5)
        dw.unpack(want)
        back = dw.arena_host()
        w.arena[:] = 0xA5
        orc.unpack(tab, len(w.shards), want)
        assert gu.first_mismatch(back, w.arena) is None
        dw.close()
    finally:
        ds.ds_config_set("grid_limit", 0)


@pytest.mark.parametrize("variant", [0, 1])
def test_repeated_launches_give_the_same_bytes(variant):
    """Thirty gathers and ten scatters in a row, each compared with the oracle: a
    result that depends on timing (a missing wait, a hazard) shows up as a
    mismatch in some of them."""
    ds, orc, gu = _mods()
    w = W.fragmentation(1500, max_bytes=1 << 19, seed=77)
    print(f"[case] repeated launches variant={variant}", flush=True)
    want, offs, tab = gu.oracle_image(w)
    ds.ds_config_set("variant", variant)
    try:
        dw = gu.DeviceWorkload(w)
        bad = [rep for rep in range(30) if gu.first_mismatch(dw.pack(), want) is not None]
        assert not bad, bad
        keep = w.arena.copy()
        w.arena[:] = 0xA5
        orc.unpack(tab, len(w.shards), want)
        for rep in range(10):
            dw.arena.fill_(0xA5)
            dw.unpack(want)
            assert gu.first_mismatch(dw.arena_host(), w.arena) is None, rep
        w.arena[:] = keep
        dw.close()
    finally:
        ds.ds_config_set("variant", 0)


def test_image_ranges_concatenate_to_the_whole():
    """Sec. V-A4: a chunk need not be a whole object -- any partition of the
    image into ranges (multiples of 16) gives the same bytes."""
    ds, orc, gu = _mods()
    w = W.fragmentation(1200, max_bytes=1 << 18, seed=55)
    want, _, _ = gu.oracle_image(w)
    dw = gu.DeviceWorkload(w)
    rng = np.random.default_rng(1)
    try:
        for trial in range(4):
            cuts = sorted(set(int(x) * 16 for x in rng.integers(0, dw.total // 16, size=int(rng.integers(1, 40)))))
            edges = [0] + cuts + [dw.total]
            print(f"[case] ranges trial={trial} n={len(edges) - 1}", flush=True)
            parts = [dw.pack(lo, hi) for lo, hi in zip(edges[:-1], edges[1:]) if hi > lo]
            got = np.concatenate(parts)
            assert gu.first_mismatch(got, want) is None, gu.first_mismatch(got, want)
        # scatter by ranges too
        dw.arena.fill_(0xA5)
        for lo, hi in zip(edges[:-1], edges[1:]):
            if hi > lo:
                dw.unpack(want, lo, hi)
        tab = orc.table(w.shards, w.arena.ctypes.data)
        for i, off in enumerate(dw.offsets):
            tab[i].file_offset = off
        w.arena[:] = 0xA5
        orc.unpack(tab, len(w.shards), want)
        assert gu.first_mismatch(dw.arena_host(), w.arena) is None
    finally:
        dw.close()


def _adhoc(arena, shards, align):
    return Workload("adhoc", align, 0, arena, shards)


def test_edge_cases_given_offsets_holes_empty_scalar_6d():
    ds, orc, gu = _mods()
    rng = np.random.default_rng(9)
    arena = rng.integers(0, 256, size=1 << 16, dtype=np.uint8)
    shards = [
        Shard("scalar", "i64", (), (), 8, 0),
        Shard("empty", "f32", (0, 5), (5, 1), 64, 1),
        Shard("six_d", "bf16", (2, 2, 2, 2, 2, 3), (400, 190, 90, 40, 16, 2), 1024, 2),
        Shard("transposed", "f32", (7, 5), (1, 9), 8192, 3),
        Shard("odd_tail", "u8", (1001,), (1,), 12001, 4),
        Shard("strided_1d", "f16", (333,), (5,), 20000, 5),
        Shard("ones", "u8", (1, 1, 13), (7, 7, 1), 30003, 6),
        Shard("rows_short", "u8", (40, 6), (9, 1), 31001, 7),
    ]
    w = _adhoc(arena, shards, 64)
    # caller-given offsets: any order, a hole at the start, a big hole in the middle
    offsets = [4096, 128, 256, 64 * 100, 64 * 300, 64 * 20, 64 * 500, 64 * 40]
    print("[case] edge cases", flush=True)
    want, offs, tab = gu.oracle_image(w, offsets=offsets)
    dw = gu.DeviceWorkload(w, offsets=offsets)
    try:
        assert dw.total == want.size
        got = dw.pack()
        assert gu.first_mismatch(got, want) is None, gu.first_mismatch(got, want)
        dw.arena.fill_(0xA5)
        dw.unpack(want)
        w.arena[:] = 0xA5
        orc.unpack(tab, len(shards), want)
        assert gu.first_mismatch(dw.arena_host(), w.arena) is None
    finally:
        dw.close()


def test_empty_table_and_all_empty_shards():
    ds, orc, gu = _mods()
    arena = np.zeros(4096, dtype=np.uint8)
    dw = gu.DeviceWorkload(_adhoc(arena, [], 256))
    assert dw.total == 0 and dw.info["n_chunks"] == 0
    ds.ds_pack(dw.plan, 0, 0, 0, 0)          # a no-op, not an error
    dw.close()
    w = _adhoc(arena, [Shard("e0", "u8", (0,), (1,), 0, 0), Shard("e1", "f32", (3, 0), (1, 1), 0, 1)], 256)
    dw = gu.DeviceWorkload(w, offsets=[0, 512])
    try:
        assert dw.total == 512                 # an empty shard still claims its offset
        got = dw.pack()
        assert not got.any() and got.size == 512
    finally:
        dw.close()


def test_range_and_argument_errors_on_device_plan():
    ds, orc, gu = _mods()
    w = W.fragmentation(10, max_bytes=4096, seed=3)
    dw = gu.DeviceWorkload(w)
    import torch
    buf = torch.zeros(dw.total + 64, dtype=torch.uint8, device="cuda")
    try:
        for lo, hi in [(16, 0), (0, dw.total + 16), (8, 32), (0, 24)]:
            with pytest.raises(ds.DsError) as e:
                ds.ds_pack(dw.plan, buf.data_ptr(), lo, hi, 0)
            assert e.value.code == ds.DS_ERANGE
        with pytest.raises(ds.DsError) as e:
            ds.ds_pack(dw.plan, buf.data_ptr() + 8, 0, dw.total, 0)
        assert e.value.code == ds.DS_EINVAL
        with pytest.raises(ds.DsError) as e:
            ds.ds_unpack(dw.plan, 0, 0, dw.total, 0)
        assert e.value.code == ds.DS_EINVAL
    finally:
        dw.close()


def test_plan_memory_check_turns_wrong_descriptors_into_errors():
    """DS_PLAN_CHECK_MEMORY: a table whose views all lie inside their allocations is accepted and packs as
    usual; views that run past the end of their allocation and a host address are refused
    with DS_EFAULT at plan time -- nothing is launched on them."""
    import torch
    ds, orc, gu = _mods()
    w = W.fragmentation(300, max_bytes=1 << 14, seed=8)
    want, _, _ = gu.oracle_image(w)
    dw = gu.DeviceWorkload(w, flags=ds.DS_PLAN_CHECK_MEMORY | ds.DS_PLAN_STRICT)
    try:
        assert gu.first_mismatch(dw.pack(), want) is None
    finally:
        dw.close()
    small = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    host = np.zeros(4096, dtype=np.uint8)
    cases = {
        "runs past the end": Shard("x", "u8", (1 << 30,), (1,), 0, 0),              # 1 GiB claimed in a 4 KiB tensor
        "rows run past the end": Shard("x", "f32", (1 << 20, 4), (1 << 12, 1), 0, 0),
    }
    for name, sh in cases.items():
        print(f"[case] memory check: {name}", flush=True)
        d = ds.make_descs([sh], small.data_ptr())
        ds.ds_layout_assign(d, 1, 256)
        with pytest.raises(ds.DsError) as e:
            ds.ds_plan_create(d, 1, 256, ds.DS_PLAN_CHECK_MEMORY)
        assert e.value.code == ds.DS_EFAULT, name
        ds.ds_plan_destroy(ds.ds_plan_create(d, 1, 256, ds.DS_PLAN_HOST_ONLY))   # the table itself is well-formed
    d = ds.make_descs([Shard("h", "u8", (4096,), (1,), 0, 0)], host.ctypes.data)
    ds.ds_layout_assign(d, 1, 256)
    with pytest.raises(ds.DsError) as e:
        ds.ds_plan_create(d, 1, 256, ds.DS_PLAN_CHECK_MEMORY)
    assert e.value.code == ds.DS_EFAULT


def test_sizes_beyond_32_bits():
    """One contiguous shard of 5 GiB (offsets inside a tile beyond 2^32) and a 2-D
    view whose rows are longer than 2^31 bytes (the 64-bit index path of the
    general path), pack and restore, whole image and whole arena."""
    ds, orc, gu = _mods()
    import torch
    GiB = 1 << 30
    big = 5 * GiB + 48                      # not a multiple of the chunk size: ends inside a chunk
    row = 2 * GiB + 4112                    # > 2^31, a multiple of 16
    pitch = row + 4096
    arena_bytes = 512 + big + 1024 + 2 * pitch
    rng = np.random.default_rng(12)
    arena = np.empty(arena_bytes, dtype=np.uint8)
    blk = rng.integers(0, 256, size=1 << 26, dtype=np.uint8)
    for lo in range(0, arena_bytes, blk.size):            # period 64 MiB, shifted per block so that
        n = min(blk.size, arena_bytes - lo)               # a displacement by the period is still seen
        arena[lo:lo + n] = np.roll(blk, lo >> 26)[:n]
    second = (512 + big + 1024 + 15) & ~15
    shards = [Shard("flat5g", "u8", (big,), (1,), 512 + 4, 0),
              Shard("long_rows", "u8", (2, row), (pitch, 1), second + 3, 1),
              Shard("tail", "i64", (3,), (1,), 8, 2)]
    w = _adhoc(arena, shards, 4096)
    print(f"[case] beyond 32 bits: arena {arena_bytes} bytes", flush=True)
    want, offs, tab = gu.oracle_image(w)
    dw = gu.DeviceWorkload(w)
    try:
        assert dw.total == want.size and dw.offsets == offs
        image = torch.full((dw.total,), 0xFF, dtype=torch.uint8, device="cuda")
        s = torch.cuda.current_stream().cuda_stream
        ds.ds_pack(dw.plan, image.data_ptr(), 0, dw.total, s)
        torch.cuda.synchronize()
        got = image.cpu().numpy()
        assert gu.first_mismatch(got, want) is None, gu.first_mismatch(got, want)
        del got
        dw.arena.fill_(0xA5)
        image.copy_(torch.from_numpy(want))
        ds.ds_unpack(dw.plan, image.data_ptr(), 0, dw.total, s)
        torch.cuda.synchronize()
        back = dw.arena_host()
        w.arena[:] = 0xA5
        orc.unpack(tab, len(shards), want)
        assert gu.first_mismatch(back, w.arena) is None, gu.first_mismatch(back, w.arena)
    finally:
        dw.close()


def test_copy_probe_copies():
    ds, orc, gu = _mods()
    import torch
    for n in (16, 16 * 1023, 16 * 1024, 16 * 1025, (64 << 20) + 48):
        src = torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.zeros(n + 64, dtype=torch.uint8, device="cuda")
        ds.ds_copy_probe(dst.data_ptr(), src.data_ptr(), n, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert torch.equal(dst[:n], src) and not dst[n:].any(), n
    with pytest.raises(ds.DsError):
        ds.ds_copy_probe(dst.data_ptr(), src.data_ptr(), 24, 0)


def test_torch_views_pack_to_what_contiguous_holds():
    """Descriptors taken straight from torch tensors (slices, a transposed matrix,
    a strided 3-D view, a scalar): the image must hold, at each shard's offset,
    the bytes of tensor.contiguous() -- the row-major order of the VIEW."""
    import torch
    import paper_2601_16956_amd as ds
    g = torch.Generator(device="cuda").manual_seed(4)
    big = torch.randn(300, 517, device="cuda", generator=g)
    half = torch.randn(64, 96, 40, device="cuda", generator=g).to(torch.bfloat16)
    ints = torch.arange(10000, device="cuda", dtype=torch.int64)
    raw = torch.randint(0, 256, (70001,), device="cuda", dtype=torch.uint8, generator=g)
    tensors = [
        big,                                  # contiguous
        big[:, 5:400],                        # column slice: rows of 395 floats, pitch 517
        big.t(),                              # transposed: inner stride 517
        half[::2, 1:90:3, :],                 # strided in two outer dimensions
        half.to(torch.float16)[3],            # contiguous 2-D slice of another dtype
        ints[7:9000:13],                      # 1-D with a stride
        raw[1:70000],                         # odd base address, odd length
        torch.tensor(3.5, device="cuda"),     # 0-D
    ]
    d = ds.make_descs_from_tensors(tensors)
    n = len(tensors)
    total = ds.ds_layout_assign(d, n, 256)
    plan = ds.ds_plan_create(d, n, 256, ds.DS_PLAN_STRICT)
    image = torch.full((total,), 0xFF, dtype=torch.uint8, device="cuda")
    s = torch.cuda.current_stream().cuda_stream
    ds.ds_pack(plan, image.data_ptr(), 0, total, s)
    torch.cuda.synchronize()
    expect = torch.zeros(total, dtype=torch.uint8, device="cuda")
    for i, t in enumerate(tensors):
        tid, dt, off, nb = ds.ds_plan_shard(plan, i)
        assert nb == t.numel() * t.element_size() and ds.ds_plan_shard_shape(plan, i) == tuple(t.shape)
        expect[off:off + nb] = t.contiguous().reshape(-1).view(torch.uint8)
    assert torch.equal(image, expect)
    # and back: wipe the tensors' parents, scatter, the views read as before
    saved = [t.clone() for t in tensors]
    for parent in (big, half, ints, raw):
        parent.zero_()
    tensors[4].zero_()
    tensors[7].zero_()
    ds.ds_unpack(plan, image.data_ptr(), 0, total, s)
    torch.cuda.synchronize()
    for t, keep in zip(tensors, saved):
        assert torch.equal(t.contiguous().reshape(-1).view(torch.uint8), keep.contiguous().reshape(-1).view(torch.uint8))
    ds.ds_plan_destroy(plan)


def test_pack_and_unpack_inside_a_hip_graph():
    """ds_pack / ds_unpack only enqueue a kernel, so a caller may capture them in a
    HIP graph; every replay (with eager work and synchronisations in between, and
    the tensors changed between replays) must give the oracle's bytes."""
    ds, orc, gu = _mods()
    import torch
    w = W.fragmentation(900, max_bytes=1 << 17, seed=83)
    print("[case] graph capture", flush=True)
    dw = gu.DeviceWorkload(w)
    n = len(w.shards)
    tab = orc.table(w.shards, w.arena.ctypes.data)
    total = orc.layout(tab, n, w.align)
    image = torch.empty(total, dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    try:
        ds.ds_pack(dw.plan, image.data_ptr(), 0, total, torch.cuda.current_stream().cuda_stream)   # warm, eager
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            ds.ds_pack(dw.plan, image.data_ptr(), 0, total, side.cuda_stream)
        for rep in range(3):
            w.arena[:] = (w.arena.astype(np.uint16) * 7 + rep + 1).astype(np.uint8)    # new tensor contents
            dw.arena.copy_(torch.from_numpy(w.arena))
            image.fill_(0xFF)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            want = orc.pack(tab, n, total)
            assert gu.first_mismatch(image.cpu().numpy(), want) is None, rep
        # the scatter, captured: image -> wiped tensors
        g2 = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g2, stream=side):
            ds.ds_unpack(dw.plan, image.data_ptr(), 0, total, side.cuda_stream)
        for rep in range(2):
            dw.arena.fill_(0xA5)
            torch.cuda.synchronize()
            g2.replay()
            torch.cuda.synchronize()
            keep = w.arena.copy()
            w.arena[:] = 0xA5
            orc.unpack(tab, n, want)
            assert gu.first_mismatch(dw.arena_host(), w.arena) is None, rep
            w.arena[:] = keep
    finally:
        del graph
        dw.close()


def _random_table(rng, arena_bytes):
    """Shards with 0..6 dimensions, extents from 0/1 up to hundreds, strides that keep the view free of
    self-overlap (built innermost first with random slack, then the dimensions are permuted, so transposed
    and interleaved layouts occur), any dtype, element-aligned bases."""
    from workloads.configs import DTYPES
    shards = []
    for i in range(int(rng.integers(1, 25))):
        dtype = list(DTYPES)[int(rng.integers(0, 5))]
        es = DTYPES[dtype][1]
        nd = int(rng.integers(0, 7))
        budget = int(2 ** rng.uniform(4, 17))             # elements, roughly
        shape = []
        for _ in range(nd):
            e = int(rng.choice([0, 1, 1, 2, 3, 5, 8, 16, 31, 64, 100, 257]))
            shape.append(min(e, max(budget, 1)))
            budget = max(budget // max(e, 1), 1)
        strides, acc = [], 1
        for e in reversed(shape):
            here = acc + int(rng.choice([0, 0, 0, 1, 3, 16]))
            strides.append(here)
            acc = here * max(e, 1)
        strides.reverse()
        perm = rng.permutation(nd) if nd and rng.random() < 0.4 else np.arange(nd)
        shape = tuple(int(shape[j]) for j in perm)
        strides = tuple(int(strides[j]) for j in perm)
        span = 1 + sum((max(e, 1) - 1) * st for e, st in zip(shape, strides))
        if span * es >= arena_bytes // 2:
            continue
        start = int(rng.integers(0, (arena_bytes - span * es) // es)) * es
        shards.append(Shard(f"r{i}", dtype, shape, strides, start, 1000 + i))
    return shards


def test_random_tables_pack_and_unpack():
    """Sixty random shard tables (see _random_table), random alignments; half of them with offsets given by
    the caller in shuffled order with holes.  Gather and scatter against the oracle, whole image, whole arena."""
    ds, orc, gu = _mods()
    rng = np.random.default_rng(2601)
    arena_bytes = 1 << 22
    for trial in range(60):
        arena = rng.integers(0, 256, size=arena_bytes, dtype=np.uint8)
        shards = _random_table(rng, arena_bytes)
        if not shards:
            continue
        align = int(2 ** rng.integers(4, 13))
        w = _adhoc(arena, shards, align)
        offsets = None
        if trial % 2:
            sizes = [int(np.prod(s.shape, dtype=np.int64)) * s.itemsize if len(s.shape) else s.itemsize for s in shards]
            order = rng.permutation(len(shards))
            at, offsets = int(rng.integers(0, 3)) * align, [0] * len(shards)
            for j in order:
                offsets[j] = at
                at = -(-(at + sizes[j]) // align) * align + int(rng.integers(0, 3)) * align
        print(f"[case] random table trial={trial} shards={len(shards)} align={align} given={offsets is not None}", flush=True)
        want, offs, tab = gu.oracle_image(w, offsets=offsets)
        dw = gu.DeviceWorkload(w, offsets=offsets)
        try:
            assert dw.total == want.size
            got = dw.pack()
            assert gu.first_mismatch(got, want) is None, (trial, gu.first_mismatch(got, want))
            if want.size:
                # shards of a table may share arena bytes; the image was gathered from ONE arena, so they
                # agree on every shared byte and the scatter is the same in whatever order it writes
                dw.arena.fill_(0)
                dw.unpack(want)
                w.arena[:] = 0
                orc.unpack(tab, len(shards), want)
                assert gu.first_mismatch(dw.arena_host(), w.arena) is None, trial
        finally:
            dw.close()


@pytest.mark.parametrize("chunk_bytes", [8192, 16384, 32768])
def test_general_path_batches_direct_pieces_and_unit_kinds(chunk_bytes):
    """A table made for the general path: thousands of 16..60-byte shards at
    16-byte alignment (hundreds of tiles per chunk: several batches of 64),
    a large view with two outer dimensions (pieces of >= 8 KiB per chunk: the
    direct path), a view with three outer dimensions and one-element runs, rows
    shorter than 16 bytes (every unit cut), and odd-sized payload tails of every
    dtype -- gathered and scattered whole and in ranges that cut chunks."""
    from workloads.configs import DTYPES
    ds, orc, gu = _mods()
    rng = np.random.default_rng(77)
    arena_bytes = 1 << 23
    arena = rng.integers(0, 256, size=arena_bytes, dtype=np.uint8)
    shards, at = [], 0

    def put(dtype, shape, strides):
        nonlocal at
        es = DTYPES[dtype][1]
        span = 1 + sum((max(e, 1) - 1) * st for e, st in zip(shape, strides))
        at = -(-at // es) * es + es * int(rng.integers(0, 3))
        shards.append(Shard(f"g{len(shards)}", dtype, tuple(shape), tuple(strides), at, 5000 + len(shards)))
        at += span * es

    names = list(DTYPES)
    for k in range(3000):                                       # tiny shards, any dtype
        dtype = names[k % 5]
        es = DTYPES[dtype][1]
        put(dtype, [max(1, int(rng.integers(16, 61)) // es)], [1])
    put("f32", [64, 96, 40], [96 * 100 + 7, 100, 1])            # two outer dimensions, 960 KB of payload
    put("u8", [30, 7, 5, 3], [7 * 5 * 3 * 8, 5 * 3 * 4, 3 * 2, 2])   # one-element runs
    put("bf16", [4000, 6], [10, 1])                             # 12-byte rows
    put("i64", [1001, 3], [5, 1])                               # 24-byte rows: most units cut
    for dtype in names:                                         # odd tails
        es = DTYPES[dtype][1]
        put(dtype, [(1 << 15) // es + 1], [1])
    assert at < arena_bytes
    w = _adhoc(arena, shards, 16)
    ds.ds_config_set("chunk_bytes", chunk_bytes)
    try:
        print(f"[case] general path table chunk_bytes={chunk_bytes} shards={len(shards)}", flush=True)
        want, offs, tab = gu.oracle_image(w)
        dw = gu.DeviceWorkload(w)
        try:
            assert dw.info["n_general_chunks"] >= 40
            got = dw.pack()
            assert gu.first_mismatch(got, want) is None, gu.first_mismatch(got, want)
            for lo, hi in ((16, 48), (4096 + 16, 3 * chunk_bytes + 32), (dw.total - chunk_bytes - 16, dw.total)):
                part = dw.pack(lo, hi)
                assert gu.first_mismatch(part, want[lo:hi]) is None, (lo, hi, gu.first_mismatch(part, want[lo:hi]))
            dw.arena.fill_(0x5A)
            dw.unpack(want)
            w.arena[:] = 0x5A
            orc.unpack(tab, len(shards), want)
            assert gu.first_mismatch(dw.arena_host(), w.arena) is None
        finally:
            dw.close()
    finally:
        ds.ds_config_set("chunk_bytes", 16384)


@pytest.mark.parametrize("block_bytes", [16384, 65536, 1 << 20])
def test_image_diff_flags_exactly_the_blocks_that_differ(block_bytes):
    """ds_image_diff against its definition (a block is flagged iff some byte of it differs) on image pairs
    with planted differences: none, one byte at the first / last position of a block, of the image, of
    the ragged last block, and many."""
    import torch
    ds, orc, gu = _mods()
    rng = np.random.default_rng(31)
    for nbytes in (16, 16384, 16384 * 3 + 4096, (5 << 20) + 16 * 37):
        base = rng.integers(0, 256, size=nbytes, dtype=np.uint8)
        n_blocks = -(-nbytes // block_bytes)
        cases = [[], [0], [nbytes - 1], [min(block_bytes, nbytes) - 1], list(rng.integers(0, nbytes, size=40))]
        if n_blocks > 1:
            cases += [[block_bytes], [block_bytes * (n_blocks - 1)], [block_bytes * (n_blocks - 1) - 1]]
        a = torch.from_numpy(base).cuda()
        for pos in cases:
            other = base.copy()
            for p in pos:
                other[p] ^= 0x01 << int(rng.integers(0, 8))
            b = torch.from_numpy(other).cuda()
            flags = torch.full((n_blocks,), 7, dtype=torch.int32, device="cuda")     # stale values must be cleared
            ds.ds_image_diff(a.data_ptr(), b.data_ptr(), nbytes, block_bytes, flags.data_ptr(),
                             torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            want = orc.image_diff(base, other, block_bytes)
            assert flags.cpu().tolist() == want, (nbytes, pos[:4])
    with pytest.raises(ds.DsError) as e:
        ds.ds_image_diff(a.data_ptr(), b.data_ptr(), nbytes, 4096, flags.data_ptr(), 0)
    assert e.value.code == ds.DS_ERANGE
    with pytest.raises(ds.DsError) as e:
        ds.ds_image_diff(a.data_ptr() + 4, b.data_ptr(), 1024, block_bytes, flags.data_ptr(), 0)
    assert e.value.code == ds.DS_EINVAL


def test_contiguous_tensors_at_every_byte_alignment():
    """Contiguous tensors whose device address is 0..15 bytes past a multiple of 16, each several chunks long:
    their interior chunks take the gather's aligned-load route (units assembled from two aligned 16-byte loads,
    the second one another lane's), first and last chunks the plain one.  Gather and scatter against the
    oracle, whole image and whole arena, at the three chunk sizes."""
    ds, orc, gu = _mods()
    rng = np.random.default_rng(1616)
    arena = rng.integers(0, 256, size=24 << 20, dtype=np.uint8)
    shards, at = [], 0
    for m in range(16):
        for dtype, es in (("u8", 1), ("bf16", 2), ("f32", 4), ("i64", 8)):
            if m % es:
                continue
            nbytes = int(rng.integers(40, 400)) * 1024 + int(rng.integers(0, 64)) * es
            start = (at + 255) // 256 * 256 + m
            shards.append(Shard(f"a{m}_{dtype}", dtype, (nbytes // es,), (1,), start, 100 * m + es))
            at = start + nbytes
    assert at < arena.size
    w = _adhoc(arena, shards, 256)
    want, offs, tab = gu.oracle_image(w)
    for chunk_bytes in (16384, 8192, 32768):
        ds.ds_config_set("chunk_bytes", chunk_bytes)
        print(f"[case] byte alignments, chunk {chunk_bytes}", flush=True)
        dw = gu.DeviceWorkload(w)
        try:
            got = dw.pack()
            assert gu.first_mismatch(got, want) is None, (chunk_bytes, gu.first_mismatch(got, want))
            dw.arena.fill_(0x5A)
            dw.unpack(want)
            keep = w.arena.copy()
            w.arena[:] = 0x5A
            orc.unpack(tab, len(shards), want)
            bad = gu.first_mismatch(dw.arena_host(), w.arena)
            w.arena[:] = keep
            assert bad is None, (chunk_bytes, bad)
        finally:
            dw.close()
            ds.ds_config_set("chunk_bytes", 16384)


def test_plans_of_mostly_general_chunks():
    """A table of thousands of tiny tensors (every 16 KiB chunk holds tile boundaries): such a plan is launched
    with five wavefronts per SIMD instead of four (variant 5 keeps four).  Both launches against the oracle,
    gather and scatter, whole image and whole arena."""
    ds, orc, gu = _mods()
    rng = np.random.default_rng(555)
    arena = rng.integers(0, 256, size=48 << 20, dtype=np.uint8)
    shards, at = [], 0
    for k in range(30000):
        dtype, es = [("u8", 1), ("bf16", 2), ("f32", 4), ("i64", 8)][k % 4]
        n = int(rng.integers(1, 1100 // es))
        start = (at + 7) // 8 * 8 + int(rng.integers(0, 8 // es)) * es
        shards.append(Shard(f"t{k}", dtype, (n,), (1,), start, k))
        at = start + n * es
    assert at < arena.size
    w = _adhoc(arena, shards, 512)
    want, offs, tab = gu.oracle_image(w)
    old_v = ds.ds_config_get("variant")
    try:
        for variant in (0, 5):
            ds.ds_config_set("variant", variant)
            print(f"[case] mostly general chunks, variant {variant}", flush=True)
            dw = gu.DeviceWorkload(w)
            try:
                assert dw.info["n_general_chunks"] * 2 > dw.info["n_chunks"]
                got = dw.pack()
                assert gu.first_mismatch(got, want) is None, (variant, gu.first_mismatch(got, want))
                dw.arena.fill_(0x5A)
                dw.unpack(want)
                keep = w.arena.copy()
                w.arena[:] = 0x5A
                orc.unpack(tab, len(shards), want)
                bad = gu.first_mismatch(dw.arena_host(), w.arena)
                w.arena[:] = keep
                assert bad is None, (variant, bad)
            finally:
                dw.close()
    finally:
        ds.ds_config_set("variant", old_v)


def test_row_views_at_every_byte_alignment():
    """2-D views whose rows start at every byte position relative to a multiple of 16 (base address, row length
    and pitch all vary; rows from 16 bytes to several chunks), each many chunks long: the lean row path with
    its unaligned 16-byte accesses and its units cut by row ends (spliced from two in-row loads in the gather,
    stored in pieces by the scatter).  Gather (whole and in ranges) and scatter against the oracle, whole image
    and whole arena, at the three chunk sizes."""
    ds, orc, gu = _mods()
    rng = np.random.default_rng(2718)
    arena = rng.integers(0, 256, size=96 << 20, dtype=np.uint8)
    shards, at = [], 0
    shapes = [(16, 24), (17, 23), (18, 27), (31, 33), (33, 48), (47, 47 * 3), (100, 150), (510, 765), (1000, 1500),
              (4094, 6141), (5504, 22016 + 2), (16384 + 6, 16384 + 38), (40000, 40002)]
    for k, (run, pitch) in enumerate(shapes):
        for dtype, es in (("u8", 1), ("bf16", 2), ("f32", 4), ("i64", 8)):
            if run % es or pitch % es:
                continue
            m = int(rng.integers(0, 16 // es)) * es if es < 16 else 0
            rows = max(3, (int(rng.integers(70, 200)) * 1024) // run)
            start = (at + 255) // 256 * 256 + m
            shards.append(Shard(f"r{k}_{dtype}", dtype, (rows, run // es), (pitch // es, 1), start, 100 * k + es))
            at = start + (rows - 1) * pitch + run
    assert at < arena.size
    w = _adhoc(arena, shards, 256)
    want, offs, tab = gu.oracle_image(w)
    for chunk_bytes in (16384, 8192, 32768):
        ds.ds_config_set("chunk_bytes", chunk_bytes)
        print(f"[case] row alignments, chunk {chunk_bytes}", flush=True)
        dw = gu.DeviceWorkload(w)
        try:
            got = dw.pack()
            assert gu.first_mismatch(got, want) is None, (chunk_bytes, gu.first_mismatch(got, want))
            for lo, hi in ((16, dw.total - 48), (dw.total // 3 // 16 * 16, dw.total // 2 // 16 * 16)):
                part = dw.pack(lo, hi)
                assert gu.first_mismatch(part, want[lo:hi]) is None, (chunk_bytes, lo, hi)
            dw.arena.fill_(0x5A)
            dw.unpack(want)
            keep = w.arena.copy()
            w.arena[:] = 0x5A
            orc.unpack(tab, len(shards), want)
            bad = gu.first_mismatch(dw.arena_host(), w.arena)
            w.arena[:] = keep
            assert bad is None, (chunk_bytes, bad)
        finally:
            dw.close()
            ds.ds_config_set("chunk_bytes", 16384)


def test_views_whose_strides_do_not_nest():
    """Views that address no element twice although a larger stride lies inside the reach of a smaller one
    (shape (3,2) with strides (2,3) addresses 0,3,2,5,4,7): the plan accepts them after writing the addresses
    out; gather and scatter against the oracle, whole image and whole arena."""
    ds, orc, gu = _mods()
    rng = np.random.default_rng(2323)
    arena = rng.integers(0, 256, size=4 << 20, dtype=np.uint8)
    shards, at = [], 0
    views = [((3, 2), (2, 3)), ((500, 2), (2, 3)), ((2, 700), (3, 2)), ((3, 4, 2), (5, 7, 1)), ((64, 3, 2), (16, 2, 3)),
             ((1 << 15, 2), (2, 3))]
    for k, (shape, strides) in enumerate(views):
        addr = [sum(i * st for i, st in zip(idx, strides)) for idx in np.ndindex(*shape)]
        assert len(set(addr)) == len(addr)                              # it is a view
        for dtype, es in (("u8", 1), ("bf16", 2), ("f32", 4), ("i64", 8)):
            start = (at + 511) // 512 * 512
            shards.append(Shard(f"v{k}_{dtype}", dtype, shape, strides, start, 10 * k + es))
            at = start + (max(addr) + 1) * es
    assert at < arena.size
    w = _adhoc(arena, shards, 64)
    want, offs, tab = gu.oracle_image(w)
    print("[case] strides that do not nest", flush=True)
    dw = gu.DeviceWorkload(w)
    try:
        got = dw.pack()
        assert gu.first_mismatch(got, want) is None, gu.first_mismatch(got, want)
        dw.arena.fill_(0x5A)
        dw.unpack(want)
        keep = w.arena.copy()
        w.arena[:] = 0x5A
        orc.unpack(tab, len(shards), want)
        bad = gu.first_mismatch(dw.arena_host(), w.arena)
        w.arena[:] = keep
        assert bad is None, bad
    finally:
        dw.close()


@pytest.mark.parametrize("block_bytes", [16384, 65536, 1 << 20])
def test_image_compress_equals_the_block_elision_oracle(block_bytes):
    """ds_image_compress against oracle/image_compress.py: flags, positions, patterns and the packed blocks,
    on images with planted constant blocks (zeros, 0xFF, a 16-byte pattern), blocks that differ from constant in
    one byte (first / last unit), a ragged last block; then the oracle's decompression of the DEVICE's output
    must give the image back."""
    import torch
    from oracle import image_compress as ic
    ds, orc, gu = _mods()
    rng = np.random.default_rng(77)
    s = torch.cuda.current_stream().cuda_stream
    for nbytes in (16, block_bytes, block_bytes * 5 + 16 * 37, block_bytes * 40):
        img = rng.integers(0, 256, size=nbytes, dtype=np.uint8)
        n_blocks = -(-nbytes // block_bytes)
        for k in range(n_blocks):
            blk = img[k * block_bytes:(k + 1) * block_bytes]
            kind = k % 6
            if kind == 0:
                blk[:] = 0
            elif kind == 1:
                blk[:] = np.tile(rng.integers(0, 256, 16, dtype=np.uint8), blk.size // 16)
            elif kind == 2 and blk.size > 16:
                blk[:] = 0xFF
                blk[blk.size - 1] = 0xFE                     # the last byte of the block
            elif kind == 3 and blk.size > 16:
                blk[:] = 0
                blk[16] = 1                                  # the first byte behind the first unit
        print(f"[case] compress nbytes={nbytes} block={block_bytes}", flush=True)
        keep_w, pos_w, pat_w, packed_w = ic.compress(img, block_bytes)
        d_img = torch.from_numpy(img).cuda()
        keep = torch.full((n_blocks,), 9, dtype=torch.int32, device="cuda")          # stale values must be cleared
        pos = torch.full((n_blocks + 1,), 9, dtype=torch.int32, device="cuda")
        pats = torch.full((n_blocks * 16,), 0xCC, dtype=torch.uint8, device="cuda")
        packed = torch.full((n_blocks * block_bytes,), 0xCC, dtype=torch.uint8, device="cuda")
        ds.ds_image_compress(d_img.data_ptr(), nbytes, block_bytes, keep.data_ptr(), pos.data_ptr(), pats.data_ptr(),
                             packed.data_ptr(), s)
        torch.cuda.synchronize()
        keep_g = keep.cpu().numpy().astype(np.uint32)
        pos_g = pos.cpu().numpy().astype(np.uint32)
        assert keep_g.tolist() == keep_w.tolist(), nbytes
        assert pos_g.tolist() == pos_w.tolist(), nbytes
        assert np.array_equal(pats.cpu().numpy().reshape(-1, 16), pat_w)
        packed_g = packed.cpu().numpy()
        for k in range(n_blocks):
            if keep_w[k]:
                length = min(block_bytes, nbytes - k * block_bytes)
                at = int(pos_w[k]) * block_bytes
                assert np.array_equal(packed_g[at:at + length], packed_w[at:at + length]), (nbytes, k)
        assert np.all(packed_g[int(pos_w[-1]) * block_bytes:] == 0xCC)                 # nothing behind the kept blocks
        back = ic.decompress(keep_g, pos_g, pats.cpu().numpy().reshape(-1, 16), packed_g, nbytes, block_bytes)
        assert np.array_equal(back, img)
    with pytest.raises(ds.DsError) as e:
        ds.ds_image_compress(d_img.data_ptr(), nbytes, 4096, keep.data_ptr(), pos.data_ptr(), pats.data_ptr(),
                             packed.data_ptr(), 0)
    assert e.value.code == ds.DS_ERANGE
