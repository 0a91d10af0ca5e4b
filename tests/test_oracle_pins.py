"""Pins for the CPU oracle: everything here checks oracle/ds_oracle.c against
something that is not the oracle -- hand-computed fixtures, closed forms,
numpy's own tobytes(), an explicit pure-Python element walk, invariants.
No GPU, no HIP library."""
import ctypes
import itertools
import json
import math
import os

import numpy as np
import pytest

import workloads as W
from oracle import ds_oracle as orc
from workloads.configs import DTYPES, Shard, Workload

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def make_workload(arena, shards, align):
    return Workload("adhoc", align, 0, arena, shards)


def oracle_image(w, offsets=None):
    tab = orc.table(w.shards, w.arena.ctypes.data)
    n = len(w.shards)
    if offsets is None:
        total = orc.layout(tab, n, w.align)
    else:
        for i, off in enumerate(offsets):
            tab[i].file_offset = off
        total = orc.image_bytes(tab, n, w.align)
    img = orc.pack(tab, n, total)
    return img, [int(tab[i].file_offset) for i in range(n)], tab


# ---------------------------------------------------------------------------
# layout (Sec. V-A5 rule (1): offsets follow from the sizes alone)
# ---------------------------------------------------------------------------

def test_itemsizes():
    L = orc.lib()
    assert [L.dso_itemsize(c) for c in range(5)] == [4, 2, 2, 8, 1]
    assert L.dso_itemsize(5) == 0


def test_layout_hand_fixture():
    """tests/golden/layout_hand.json: sizes and alignments worked out by hand."""
    with open(os.path.join(GOLDEN, "layout_hand.json")) as f:
        cases = json.load(f)["cases"]
    for case in cases:
        arena = np.zeros(1 << 16, dtype=np.uint8)
        shards = [Shard(f"s{i}", "u8", (b,), (1,), 0, i) for i, b in enumerate(case["bytes"])]
        tab = orc.table(shards, arena.ctypes.data)
        total = orc.layout(tab, len(shards), case["align"])
        assert [int(tab[i].file_offset) for i in range(len(shards))] == case["offsets"], case
        assert total == case["total"], case


@pytest.mark.parametrize("align", [16, 256, 512, 4096])
def test_layout_closed_form_and_invariants(align):
    rng = np.random.default_rng(7)
    sizes = [int(x) for x in rng.integers(0, 5000, size=200)]
    arena = np.zeros(8192, dtype=np.uint8)
    shards = [Shard(f"s{i}", "u8", (b,), (1,), 0, i) for i, b in enumerate(sizes)]
    tab = orc.table(shards, arena.ctypes.data)
    n = len(shards)
    total = orc.layout(tab, n, align)
    offs = [int(tab[i].file_offset) for i in range(n)]
    # closed form: off_i = sum_{k<i} ceil(b_k / A) * A
    acc = 0
    for off, b in zip(offs, sizes):
        assert off == acc
        acc += -(-b // align) * align
    assert total == acc
    assert all(off % align == 0 for off in offs)
    assert total - sum(sizes) == sum((-b) % align for b in sizes)          # only declared padding
    assert all((-b) % align < align for b in sizes)
    assert orc.check_layout(tab, n, align, total, strict=True) == orc.OK
    assert orc.image_bytes(tab, n, align) == total


def test_check_layout_detects_each_violation():
    arena = np.zeros(4096, dtype=np.uint8)
    shards = [Shard("a", "u8", (100,), (1,), 0, 0), Shard("b", "u8", (100,), (1,), 0, 1)]
    tab = orc.table(shards, arena.ctypes.data)
    tab[0].file_offset, tab[1].file_offset = 0, 256
    assert orc.check_layout(tab, 2, 256, 512, strict=True) == orc.OK
    tab[1].file_offset = 64                               # inside shard a
    assert orc.check_layout(tab, 2, 64, 512) == orc.OVERLAP
    tab[1].file_offset = 260                              # not a multiple of 256
    assert orc.check_layout(tab, 2, 256, 512) == orc.BAD_ALIGN
    tab[1].file_offset = 512                              # a whole 256-block is in no shard
    assert orc.check_layout(tab, 2, 256, 768, strict=True) == orc.GAP
    assert orc.check_layout(tab, 2, 256, 768, strict=False) == orc.OK
    assert orc.check_layout(tab, 2, 256, 600) == orc.OUT_OF_IMAGE


# ---------------------------------------------------------------------------
# image bytes
# ---------------------------------------------------------------------------

def test_image_hand_fixture():
    """tests/golden/image_hand.json: a 32-byte arena 0..31 and three shards,
    expected image written out by hand."""
    with open(os.path.join(GOLDEN, "image_hand.json")) as f:
        g = json.load(f)
    arena = np.array(g["arena"], dtype=np.uint8)
    shards = [Shard(s["name"], s["dtype"], tuple(s["shape"]), tuple(s["strides"]), s["byte_offset"], i)
              for i, s in enumerate(g["shards"])]
    w = make_workload(arena, shards, g["align"])
    img, offs, _ = oracle_image(w)
    assert offs == g["offsets"]
    assert img.tolist() == g["image"]


def test_contiguous_shards_are_numpy_tobytes():
    """Special case that reduces to a library routine: a contiguous shard's
    bytes in the image are the parent's bytes (numpy slicing + tobytes)."""
    w = W.fragmentation(300, max_bytes=1 << 16, strided_fraction=0.0, seed=11)
    img, offs, _ = oracle_image(w)
    covered = np.zeros(img.size, dtype=bool)
    for s, off in zip(w.shards, offs):
        want = w.arena[s.byte_offset:s.byte_offset + s.nbytes].tobytes()
        assert img[off:off + s.nbytes].tobytes() == want, s.name
        covered[off:off + s.nbytes] = True
    assert not img[~covered].any()                       # padding is 0x00
    assert covered.sum() == w.payload_bytes              # total bytes == sum of shard bytes


def _index_encoded(dtype, span, rng):
    """Parent whose element i holds a value that encodes i (unique per i)."""
    _, itemsize, npdt = DTYPES[dtype]
    if dtype == "u8":
        assert span <= 256
        return np.arange(span, dtype=np.uint8)
    if dtype in ("bf16", "f16"):
        assert span <= 65536
        return np.arange(span, dtype=np.uint16)
    if dtype == "f32":
        return np.arange(span, dtype=np.uint32).view(np.float32)
    return np.arange(span, dtype=np.int64) + (1 << 40)


@pytest.mark.parametrize("dtype", list(DTYPES))
def test_strided_views_index_encoding(dtype):
    """Closed form, no copy code: if parent element i holds the number i, the
    image of a view must hold  sum_j k_j*stride_j  at rank r(k) -- computed
    here with broadcasting of index ranges, never by moving bytes."""
    rng = np.random.default_rng(5)
    _, itemsize, npdt = DTYPES[dtype]
    cases = [((4, 6), (9, 1)), ((3, 2, 4), (40, 12, 1)), ((5,), (3,)), ((2, 3), (1, 2)),
             ((2, 1, 3, 2), (50, 7, 6, 2)), ((7, 3), (3, 1)), ((1,), (1,)), ((2, 2, 2, 2, 2, 2), (64, 32, 16, 8, 4, 1))]
    for shape, strides in cases:
        span = 1 + sum((e - 1) * st for e, st in zip(shape, strides))
        lead = 3
        parent = _index_encoded(dtype, span + lead, rng)
        arena = parent.view(np.uint8).copy()
        shard = Shard("v", dtype, shape, strides, lead * itemsize, 0)
        w = make_workload(arena, [shard], 64)
        img, offs, _ = oracle_image(w)
        idx = np.zeros(shape, dtype=np.int64)
        for j, (e, st) in enumerate(zip(shape, strides)):
            sh = [1] * len(shape)
            sh[j] = e
            idx = idx + (np.arange(e, dtype=np.int64) * st).reshape(sh)
        want_index = (idx + lead).reshape(-1)              # row-major rank order
        got = img[:shard.nbytes].view(npdt)
        want = _index_encoded(dtype, span + lead, rng)[want_index]
        assert got.tobytes() == want.tobytes(), (dtype, shape, strides)
        assert not img[shard.nbytes:].any()


def _python_walk(arena, shard, off, image):
    """The definition, element by element, in plain Python."""
    es = shard.itemsize
    r = 0
    for k in itertools.product(*[range(e) for e in shard.shape]):
        pos = shard.byte_offset + es * sum(kj * st for kj, st in zip(k, shard.strides))
        image[off + r * es: off + (r + 1) * es] = arena[pos:pos + es]
        r += 1


def test_brute_force_tiny_inputs():
    rng = np.random.default_rng(3)
    for trial in range(40):
        arena = rng.integers(0, 256, size=4096, dtype=np.uint8)
        shards = []
        for i in range(int(rng.integers(1, 6))):
            dtype = list(DTYPES)[int(rng.integers(0, 5))]
            es = DTYPES[dtype][1]
            nd = int(rng.integers(0, 4))
            shape = tuple(int(x) for x in rng.integers(0 if trial % 5 == 0 else 1, 5, size=nd))
            # strides: row-major with random slack so views do not self-overlap
            strides, acc = [], 1
            for e in reversed(shape):
                acc_here = acc + int(rng.integers(0, 3))
                strides.append(acc_here)
                acc = acc_here * max(e, 1)
            strides = tuple(reversed(strides))
            span = 1 + sum((max(e, 1) - 1) * st for e, st in zip(shape, strides))
            start = int(rng.integers(0, (4096 - span * es) // es)) * es
            shards.append(Shard(f"t{i}", dtype, shape, strides, start, i))
        w = make_workload(arena, shards, int(2 ** rng.integers(4, 9)))
        img, offs, _ = oracle_image(w)
        want = np.zeros(img.size, dtype=np.uint8)
        for s, off in zip(shards, offs):
            _python_walk(arena, s, off, want)
        assert img.tobytes() == want.tobytes(), trial


@pytest.mark.parametrize("maker", [
    lambda: W.tiny_gpt(),
    lambda: W.fragmentation(1500, max_bytes=1 << 17, seed=21),
    lambda: W.llama_rank("mini", 128, 352, 4, 2, 512, 2, 4, 8, seed=5, workers=1),
])
def test_c_loops_match_numpy_twin(maker):
    w = maker()
    img, offs, tab = oracle_image(w)
    assert orc.check_layout(tab, len(w.shards), w.align, img.size, strict=True) == orc.OK
    twin = orc.twin_pack(w, offs, img.size)
    assert img.tobytes() == twin.tobytes()


def test_given_offsets_any_order_and_zero_fill():
    """Offsets may come from the caller, in any order; holes are zero."""
    arena = np.arange(256, dtype=np.uint8)
    shards = [Shard("a", "u8", (10,), (1,), 0, 0), Shard("b", "u8", (6,), (1,), 100, 1),
              Shard("c", "u8", (0,), (1,), 50, 2)]
    w = make_workload(arena, shards, 16)
    img, offs, _ = oracle_image(w, offsets=[64, 0, 32])
    assert img.size == 80
    want = np.zeros(80, dtype=np.uint8)
    want[64:74] = np.arange(10)
    want[0:6] = np.arange(100, 106)
    assert img.tolist() == want.tolist()


def test_pack_overwrites_stale_image_bytes():
    w = W.fragmentation(50, max_bytes=4096, seed=2)
    tab = orc.table(w.shards, w.arena.ctypes.data)
    n = len(w.shards)
    total = orc.layout(tab, n, w.align)
    clean = orc.pack(tab, n, total).copy()
    dirty = np.full(total, 0xFF, dtype=np.uint8)
    orc.pack(tab, n, total, out=dirty)
    assert dirty.tobytes() == clean.tobytes()


def test_threads_give_the_same_image():
    w = W.fragmentation(400, max_bytes=1 << 16, seed=9)
    tab = orc.table(w.shards, w.arena.ctypes.data)
    n = len(w.shards)
    total = orc.layout(tab, n, w.align)
    one = orc.pack(tab, n, total).copy()
    for th in (2, 3, 8):
        many = np.full(total, 0x5A, dtype=np.uint8)
        orc.pack(tab, n, total, threads=th, out=many)
        assert many.tobytes() == one.tobytes()


# ---------------------------------------------------------------------------
# unpack
# ---------------------------------------------------------------------------

def _addressed_mask(w):
    """Bytes of the arena addressed by any shard, by explicit enumeration."""
    mask = np.zeros(w.arena.size, dtype=bool)
    for s in w.shards:
        if s.numel == 0:
            continue
        idx = np.zeros(s.shape, dtype=np.int64)
        for j, (e, st) in enumerate(zip(s.shape, s.strides)):
            sh = [1] * len(s.shape)
            sh[j] = e
            idx = idx + (np.arange(e, dtype=np.int64) * st).reshape(sh)
        start = s.byte_offset + idx.reshape(-1) * s.itemsize
        for b in range(s.itemsize):
            mask[start + b] = True
    return mask


@pytest.mark.parametrize("maker", [
    lambda: W.tiny_gpt(),
    lambda: W.fragmentation(600, max_bytes=1 << 15, seed=33),
])
def test_unpack_roundtrip_and_sentinel(maker):
    w = maker()
    img, offs, tab = oracle_image(w)
    n = len(w.shards)
    mask = _addressed_mask(w)
    original = w.arena.copy()
    # wipe: sentinel everywhere, then restore from the image
    w.arena[:] = 0xA5
    orc.unpack(tab, n, img)
    assert (w.arena[mask] == original[mask]).all()          # unpack(pack(x)) == x
    assert (w.arena[~mask] == 0xA5).all()                   # nothing else written
    # pack(unpack(img)) == img for an image with zero padding
    again = orc.pack(tab, n, img.size)
    assert again.tobytes() == img.tobytes()


def test_unpack_of_foreign_image_then_pack_returns_it():
    w = W.fragmentation(200, max_bytes=1 << 14, seed=4)
    tab = orc.table(w.shards, w.arena.ctypes.data)
    n = len(w.shards)
    total = orc.layout(tab, n, w.align)
    rng = np.random.default_rng(0)
    img = rng.integers(0, 256, size=total, dtype=np.uint8)
    payload = np.zeros(total, dtype=bool)
    for i, s in enumerate(w.shards):
        payload[tab[i].file_offset: tab[i].file_offset + s.nbytes] = True
    img[~payload] = 0
    orc.unpack(tab, n, img)
    assert orc.pack(tab, n, total).tobytes() == img.tobytes()


# ---------------------------------------------------------------------------
# generator realism (Sec. VI-D last paragraph; Table I)
# ---------------------------------------------------------------------------

def test_tiny_gpt_shape():
    w = W.tiny_gpt()
    assert len(w.shards) == 118
    assert w.payload_bytes == 1907712 * 14 + 8 + 64
    sliced = [s for s in w.shards if len(s.shape) == 3]
    assert len(sliced) == 2 * 2 * 4 and all(s.shape[2] == 128 and s.strides[1] == 256 for s in sliced)


def test_llama_rank_structure_small():
    w = W.llama_rank("mini", 128, 352, 4, 2, 512, 2, 4, 8, seed=5, workers=1)
    assert len(w.shards) == 2 * 9 + 1 + 3
    n = w.notes["n_params_rank"]
    bf16 = sum(s.nbytes for s in w.shards if s.dtype == "bf16")
    f32 = sum(s.nbytes for s in w.shards if s.dtype == "f32")
    assert bf16 == 2 * n and f32 == 3 * 4 * n // 8
    # at DP=1 the ratio would be 2 : 12 bytes per parameter (Table I: 13 GB : 82 GB)
    assert math.isclose((f32 * 8) / bf16, 6.0)


def test_image_diff_by_brute_force():
    """The block comparison, byte by byte in plain Python, on small random pairs."""
    rng = np.random.default_rng(8)
    for trial in range(50):
        n = int(rng.integers(1, 200))
        block = int(rng.integers(1, 40))
        a = rng.integers(0, 4, size=n, dtype=np.uint8)
        b = a.copy()
        for p in rng.integers(0, n, size=int(rng.integers(0, 4))):
            b[p] ^= 1
        want = []
        for lo in range(0, n, block):
            flag = 0
            for i in range(lo, min(lo + block, n)):
                if a[i] != b[i]:
                    flag = 1
            want.append(flag)
        assert orc.image_diff(a, b, block) == want
        assert len(want) == -(-n // block)


def test_image_compress_block_elision_by_hand_and_by_brute_force():
    """The block-elision oracle (oracle/image_compress.py): a hand-made image; flags against a byte loop on
    random images with planted constant, periodic and almost-constant blocks; decompress(compress(x)) == x;
    the position table is the running count of kept blocks."""
    from oracle import image_compress as ic
    # by hand: 4 blocks of 32 bytes: zeros | 0..31 | a 16-byte pattern twice | the pattern, last byte changed
    pat = bytes(range(100, 116))
    img = np.frombuffer(bytes(32) + bytes(range(32)) + pat + pat + pat + pat[:15] + b"\x00", dtype=np.uint8).copy()
    keep, pos, patterns, packed = ic.compress(img, 32)
    assert keep.tolist() == [0, 1, 0, 1] and pos.tolist() == [0, 0, 1, 1, 2]
    assert patterns[0].tolist() == [0] * 16 and bytes(patterns[2]) == pat and patterns[1].tolist() == list(range(16))
    assert bytes(packed) == bytes(range(32)) + pat + pat[:15] + b"\x00"
    assert ic.compressed_bytes(keep, 32) == 2 * 32 + 4 * 20
    assert np.array_equal(ic.decompress(keep, pos, patterns, packed, img.size, 32), img)
    # a period of 8 divides 16: constant; a period of 32 does not
    p8 = np.tile(np.arange(8, dtype=np.uint8), 8)
    p32 = np.tile(np.arange(32, dtype=np.uint8), 2)
    assert ic.compress(p8, 64)[0].tolist() == [0] and ic.compress(p32, 64)[0].tolist() == [1]
    rng = np.random.default_rng(11)
    for trial in range(30):
        block = int(rng.choice([16, 48, 64, 256, 1024]))
        n = int(rng.integers(1, 40)) * 16 * int(rng.integers(1, 9))
        img = rng.integers(0, 256, n, dtype=np.uint8)
        for k in range(-(-n // block)):
            kind = rng.integers(0, 4)
            blk = img[k * block:(k + 1) * block]
            if kind == 0:
                blk[:] = int(rng.integers(0, 2)) * 255
            elif kind == 1:
                blk[:] = np.tile(rng.integers(0, 256, 16, dtype=np.uint8), -(-blk.size // 16))[:blk.size]
            elif kind == 2 and blk.size > 16:
                blk[:] = 7
                blk[int(rng.integers(16, blk.size))] = 8     # one byte off, not in the first unit
        keep, pos, patterns, packed = ic.compress(img, block)
        for k in range(keep.size):                            # the definition, byte by byte
            blk = img[k * block:(k + 1) * block]
            const = all(blk[i] == blk[i % 16] for i in range(blk.size))
            assert keep[k] == (0 if const else 1), (trial, k)
            assert pos[k + 1] == pos[k] + keep[k]
            assert bytes(patterns[k]) == bytes(blk[:16])
        assert packed.size == int(pos[-1]) * block
        assert np.array_equal(ic.decompress(keep, pos, patterns, packed, n, block), img), trial
