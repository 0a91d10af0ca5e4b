"""The synthetic shard sets: what one GPU holds when a checkpoint is requested.

They stand in for the DeepSpeed/Megatron checkpoints of the paper's evaluation
(Sec. VI-C: BLOOM-3B and Llama 7B..70B, TP x PP x ZeRO-1).  Only what matters to
a byte mover is reproduced: how many shards there are, their dtypes, sizes,
strides and address alignment (Sec. IV-C, Table I: 2-byte parameters next to
4-byte optimizer state, many independently owned shards per rank), and the
value distribution named for each configuration.

Everything is a pure function of the seed.  Parents (the allocations a shard
view points into) are carved out of one byte arena at 512-byte granularity,
the granularity of the PyTorch device allocator; bytes between parents hold
0xEE and belong to no shard.
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Callable, List, Optional, Sequence, Tuple

import numpy as np

# name -> (interface code, itemsize, numpy storage dtype)
DTYPES = {
    "f32": (0, 4, np.float32),
    "bf16": (1, 2, np.uint16),
    "f16": (2, 2, np.uint16),
    "i64": (3, 8, np.int64),
    "u8": (4, 1, np.uint8),
}

BASE_SEED = 20260116956
ARENA_GRANULE = 512
GAP_BYTE = 0xEE


@dataclass
class Shard:
    """One view: element (0,..,0) sits `byte_offset` bytes into the arena."""
    name: str
    dtype: str
    shape: Tuple[int, ...]
    strides: Tuple[int, ...]          # in elements
    byte_offset: int
    tensor_id: int

    @property
    def itemsize(self) -> int:
        return DTYPES[self.dtype][1]

    @property
    def numel(self) -> int:
        return int(math.prod(self.shape))

    @property
    def nbytes(self) -> int:
        return self.numel * self.itemsize


@dataclass
class Workload:
    name: str
    align: int
    seed: int
    arena: np.ndarray                  # uint8, the host mirror of device memory
    shards: List[Shard]
    notes: dict = field(default_factory=dict)

    @property
    def payload_bytes(self) -> int:
        return sum(s.nbytes for s in self.shards)


# ----------------------------------------------------------------------------
# arena construction
# ----------------------------------------------------------------------------

@dataclass
class _Parent:
    offset: int
    numel: int
    dtype: str
    dist: str          # 'uniform' | 'normal' | 'bits' | 'const:<int>'


class _Builder:
    def __init__(self, seed: int):
        self.seed = seed
        self.size = 0
        self.parents: List[_Parent] = []
        self.shards: List[Shard] = []

    def parent(self, numel: int, dtype: str, dist: str) -> int:
        """Reserve an allocation of `numel` elements; returns its arena offset."""
        off = self.size
        nbytes = numel * DTYPES[dtype][1]
        self.parents.append(_Parent(off, numel, dtype, dist))
        self.size = off + ((max(nbytes, 1) + ARENA_GRANULE - 1) // ARENA_GRANULE) * ARENA_GRANULE
        return off

    def shard(self, name: str, dtype: str, shape: Sequence[int], strides: Sequence[int],
              byte_offset: int, tensor_id: int) -> None:
        self.shards.append(Shard(name, dtype, tuple(int(x) for x in shape),
                                 tuple(int(x) for x in strides), int(byte_offset), int(tensor_id)))

    def contiguous(self, name: str, dtype: str, shape: Sequence[int], dist: str, tensor_id: int) -> None:
        numel = int(math.prod(shape))
        off = self.parent(numel, dtype, dist)
        strides = []
        acc = 1
        for extent in reversed(shape):
            strides.append(acc)
            acc *= extent
        self.shard(name, dtype, shape, tuple(reversed(strides)), off, tensor_id)

    def build(self, name: str, align: int, workers: Optional[int] = None, notes: Optional[dict] = None) -> Workload:
        arena = np.full(self.size, GAP_BYTE, dtype=np.uint8)
        order = sorted(range(len(self.parents)), key=lambda i: -self.parents[i].numel)

        def fill(i: int) -> None:
            _fill_parent(arena, self.parents[i], np.random.SeedSequence([self.seed, i]))

        if workers is None:
            workers = 8
        if workers <= 1 or len(order) < 2:
            for i in order:
                fill(i)
        else:
            with ThreadPoolExecutor(max_workers=workers) as pool:
                list(pool.map(fill, order))
        return Workload(name, align, self.seed, arena, self.shards, notes or {})


_CHUNK = 1 << 22


def _to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit pattern, round to nearest even (finite inputs)."""
    b = x.view(np.uint32)
    return ((b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)


def _fill_parent(arena: np.ndarray, p: _Parent, ss: np.random.SeedSequence) -> None:
    _, itemsize, npdt = DTYPES[p.dtype]
    if p.numel == 0:
        return
    rng = np.random.Generator(np.random.PCG64(ss))
    view = arena[p.offset:p.offset + p.numel * itemsize].view(npdt)
    if p.dist.startswith("const:"):
        view[:] = int(p.dist.split(":")[1])
        return
    if p.dist == "bits":
        raw = arena[p.offset:p.offset + p.numel * itemsize]
        for lo in range(0, raw.size, _CHUNK * 8):
            hi = min(raw.size, lo + _CHUNK * 8)
            words = rng.bit_generator.random_raw((hi - lo + 7) // 8).astype(np.uint64, copy=False)
            raw[lo:hi] = words.view(np.uint8)[:hi - lo]
        return
    for lo in range(0, p.numel, _CHUNK):
        hi = min(p.numel, lo + _CHUNK)
        if p.dist == "uniform":
            x = rng.random(hi - lo, dtype=np.float32) * np.float32(2.0) - np.float32(1.0)
        elif p.dist == "normal":
            x = rng.standard_normal(hi - lo, dtype=np.float32) * np.float32(0.02)
        else:
            raise ValueError(p.dist)
        if p.dtype == "f32":
            view[lo:hi] = x
        elif p.dtype == "bf16":
            view[lo:hi] = _to_bf16_bits(x)
        elif p.dtype == "f16":
            view[lo:hi] = x.astype(np.float16).view(np.uint16)
        else:
            raise ValueError(f"{p.dist} values for {p.dtype}")


# ----------------------------------------------------------------------------
# configuration 1: tiny GPT-style state
# ----------------------------------------------------------------------------

def tiny_gpt(seed: int = BASE_SEED + 1, layers: int = 2, hidden: int = 256, ffn: int = 1024,
             vocab: int = 1024, positions: int = 1024, align: int = 256) -> Workload:
    """2 layers, hidden 256, 4 heads, FFN 1024, vocab 1024; every tensor four
    times (bf16 parameter, fp32 master, fp32 Adam m, fp32 Adam v), one int64
    step counter, one 64-byte opaque RNG blob.  Weights are [in, out].  Half of
    the weight matrices of a layer (qkv, fc1) are held as "every other
    128-column block" views: for a matrix [R, C] that is the 3-D view of shape
    [R, C/256, 128] with strides [C, 256, 1], what TP=2 rank 0 would own.
    Values uniform in [-1, 1]."""
    b = _Builder(seed)
    tensors: List[Tuple[str, Tuple[int, ...], bool]] = [
        ("wte", (vocab, hidden), False), ("wpe", (positions, hidden), False)]
    for l in range(layers):
        p = f"h{l}."
        tensors += [
            (p + "ln1.w", (hidden,), False), (p + "ln1.b", (hidden,), False),
            (p + "qkv.w", (hidden, 3 * hidden), True), (p + "qkv.b", (3 * hidden,), False),
            (p + "proj.w", (hidden, hidden), False), (p + "proj.b", (hidden,), False),
            (p + "ln2.w", (hidden,), False), (p + "ln2.b", (hidden,), False),
            (p + "fc1.w", (hidden, ffn), True), (p + "fc1.b", (ffn,), False),
            (p + "fc2.w", (ffn, hidden), False), (p + "fc2.b", (hidden,), False),
        ]
    tensors += [("lnf.w", (hidden,), False), ("lnf.b", (hidden,), False), ("lm_head", (hidden, vocab), False)]
    for copy, dtype in (("param", "bf16"), ("master", "f32"), ("adam_m", "f32"), ("adam_v", "f32")):
        for tid, (name, shape, sliced) in enumerate(tensors):
            full = f"{copy}.{name}"
            if sliced:
                rows, cols = shape
                assert cols % 256 == 0
                off = b.parent(rows * cols, dtype, "uniform")
                b.shard(full, dtype, (rows, cols // 256, 128), (cols, 256, 1), off, tid)
            else:
                b.contiguous(full, dtype, shape, "uniform", tid)
    b.contiguous("step", "i64", (1,), "const:1000", len(tensors))
    b.contiguous("rng", "u8", (64,), "bits", len(tensors) + 1)
    return b.build("tiny_gpt", align, workers=1)


# ----------------------------------------------------------------------------
# configurations 2 and 4: one rank of a Llama-style model under TP x PP x ZeRO-1
# ----------------------------------------------------------------------------

def llama_rank(name: str, hidden: int, ffn: int, heads: int, kv_heads: int, vocab: int,
               layers_local: int, tp: int, dp: int, tp_rank: int = 1, dp_rank: int = 1,
               align: int = 4096, seed: int = BASE_SEED + 2, workers: Optional[int] = None) -> Workload:
    """First pipeline stage of a Llama-style model: `layers_local` layers and
    the vocabulary-parallel embedding slice.  Weights are [out, in].
    Column-parallel weights (q, k, v, gate, up, embedding) are row blocks and
    so contiguous.  Row-parallel weights (o, down) are sliced along `in`: a 2-D
    view [out, in/tp] with strides [in, 1] into the full [out, in] parent,
    starting at column tp_rank*in/tp.  Norm vectors are replicated.  ZeRO-1:
    fp32 master, Adam m and Adam v are each ONE flat tensor, the dp_rank-th of
    dp equal slices of the flattened fp32 buffer of this rank's N parameters.
    Only a window of that buffer (the slice and 1024 neighbouring elements on
    each side) is materialised.  Values normal(0, 0.02)."""
    head_dim = hidden // heads
    q_rows = hidden // tp
    kv_rows = kv_heads * head_dim // tp
    ffn_loc = ffn // tp
    b = _Builder(seed)
    tid = 0
    n_params = 0

    def col(nm: str, shape: Tuple[int, ...]) -> None:
        nonlocal tid, n_params
        b.contiguous(nm, "bf16", shape, "normal", tid)
        n_params += int(math.prod(shape))
        tid += 1

    def row(nm: str, out: int, inner: int) -> None:
        nonlocal tid, n_params
        off = b.parent(out * inner, "bf16", "normal")
        width = inner // tp
        b.shard(nm, "bf16", (out, width), (inner, 1), off + tp_rank * width * 2, tid)
        n_params += out * width
        tid += 1

    col("embed", (vocab // tp, hidden))
    for l in range(layers_local):
        p = f"layers.{l}."
        col(p + "input_norm", (hidden,))
        col(p + "q", (q_rows, hidden))
        col(p + "k", (kv_rows, hidden))
        col(p + "v", (kv_rows, hidden))
        row(p + "o", hidden, hidden)
        col(p + "post_norm", (hidden,))
        col(p + "gate", (ffn_loc, hidden))
        col(p + "up", (ffn_loc, hidden))
        row(p + "down", hidden, ffn)
    assert n_params % dp == 0, (n_params, dp)
    part = n_params // dp
    guard = 1024
    for nm in ("fp32_master", "adam_m", "adam_v"):
        off = b.parent(part + 2 * guard, "f32", "normal")
        b.shard(f"zero1.{nm}", "f32", (part,), (1,), off + guard * 4, tid)
        tid += 1
    return b.build(name, align, workers=workers,
                   notes={"n_params_rank": n_params, "zero_partition_elems": part,
                          "tp": tp, "dp": dp, "tp_rank": tp_rank, "dp_rank": dp_rank})


def llama_7b_rank(seed: int = BASE_SEED + 2, workers: Optional[int] = None) -> Workload:
    """Llama-style 7B (32 layers, hidden 4096, FFN 11008, 32 heads, vocab
    32000) at TP=4, PP=4, ZeRO-1 with DP=8: 8 layers, 76 shards."""
    return llama_rank("llama7b_tp4_pp4_dp8", 4096, 11008, 32, 32, 32000, 8, 4, 8, seed=seed, workers=workers)


def llama_70b_rank(seed: int = BASE_SEED + 4, workers: Optional[int] = None) -> Workload:
    """Llama-2-70B shape (80 layers, hidden 8192, FFN 28672, 64 heads, 8 KV
    heads, vocab 32000) at TP=8, PP=4, ZeRO-1 with DP=8: 20 layers, 184 shards."""
    return llama_rank("llama70b_tp8_pp4_dp8", 8192, 28672, 64, 8, 32000, 20, 8, 8, seed=seed, workers=workers)


# ----------------------------------------------------------------------------
# configuration 3: fragmentation stress
# ----------------------------------------------------------------------------

def fragmentation(n_shards: int = 20000, min_bytes: int = 64, max_bytes: int = 4 << 20,
                  strided_fraction: float = 0.30, align: int = 512,
                  seed: int = BASE_SEED + 3, workers: Optional[int] = None) -> Workload:
    """Independent shards, byte sizes log-uniform in [min_bytes, max_bytes],
    dtype uniform over the five, `strided_fraction` of them 2-D views whose row
    stride is 1.5x the row length, every parent entered at a random element
    offset of 0..7 so that base addresses have every residue.  Values are
    uniform random bits (so floats include NaN and Inf patterns)."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 0xF2A6])))
    names = list(DTYPES)
    b = _Builder(seed)
    lo, hi = math.log(min_bytes), math.log(max_bytes)
    for i in range(n_shards):
        s = math.exp(rng.uniform(lo, hi))
        dtype = names[int(rng.integers(0, len(names)))]
        itemsize = DTYPES[dtype][1]
        strided = bool(rng.random() < strided_fraction)
        shift = int(rng.integers(0, 8))
        n = max(1, int(s) // itemsize)
        if strided:
            c = 2 * max(1, int(round(math.sqrt(n) / 2)))
            r = max(1, n // c)
            pitch = 3 * c // 2
            span = (r - 1) * pitch + c
            off = b.parent(span + shift, dtype, "bits")
            b.shard(f"frag{i}", dtype, (r, c), (pitch, 1), off + shift * itemsize, i)
        else:
            off = b.parent(n + shift, dtype, "bits")
            b.shard(f"frag{i}", dtype, (n,), (1,), off + shift * itemsize, i)
    return b.build(f"fragmentation_{n_shards}", align, workers=workers)


def by_name(name: str, workers: Optional[int] = None) -> Workload:
    """The configurations by the names the benchmark and the tests use."""
    if name == "tiny_gpt":
        return tiny_gpt()
    if name == "llama7b":
        return llama_7b_rank(workers=workers)
    if name == "fragmentation":
        return fragmentation(workers=workers)
    if name == "llama70b":
        return llama_70b_rank(workers=workers)
    raise KeyError(name)
