"""Helpers of the GPU parity tests: run a workload through the HIP library
(via the C ABI binding) and through the CPU oracle, on the same bytes."""
import ctypes

import numpy as np

import paper_2601_16956_amd as ds
from oracle import ds_oracle as orc


def oracle_image(w, offsets=None):
    tab = orc.table(w.shards, w.arena.ctypes.data)
    n = len(w.shards)
    if offsets is None:
        total = orc.layout(tab, n, w.align)
    else:
        for i, off in enumerate(offsets):
            tab[i].file_offset = off
        total = orc.image_bytes(tab, n, w.align)
    img = orc.pack(tab, n, total, threads=8)
    return img, [int(tab[i].file_offset) for i in range(n)], tab


class DeviceWorkload:
    """The workload's arena uploaded to the GPU + a plan over it."""

    def __init__(self, w, offsets=None, flags=0, arena_fill=None):
        import torch
        self.torch = torch
        self.w = w
        if arena_fill is None:
            self.arena = torch.from_numpy(w.arena).to("cuda")
        else:
            self.arena = torch.full((w.arena.size,), arena_fill, dtype=torch.uint8, device="cuda")
        self.n = len(w.shards)
        self.descs = ds.make_descs(w.shards, self.arena.data_ptr())
        if offsets is None:
            self.total = ds.ds_layout_assign(self.descs, self.n, w.align)
        else:
            for i, off in enumerate(offsets):
                self.descs[i].file_offset = off
            self.total = None
        # every plan of the GPU tests is made with the memory check: a generator or a test that describes memory
        # it does not own is then an error here, not a fault in a kernel
        self.plan = ds.ds_plan_create(self.descs, self.n, w.align, flags | ds.DS_PLAN_CHECK_MEMORY)
        self.info = ds.ds_plan_info(self.plan)
        if self.total is None:
            self.total = self.info["total_bytes"]
        assert self.total == self.info["total_bytes"]
        self.offsets = [int(self.descs[i].file_offset) for i in range(self.n)]

    def pack(self, lo=0, hi=None, fill=0xFF):
        torch = self.torch
        hi = self.total if hi is None else hi
        out = torch.full((max(hi - lo, 16),), fill, dtype=torch.uint8, device="cuda")
        ds.ds_pack(self.plan, out.data_ptr(), lo, hi, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        return out[:hi - lo].cpu().numpy()

    def unpack(self, image: np.ndarray, lo=0, hi=None):
        torch = self.torch
        hi = self.total if hi is None else hi
        src = torch.from_numpy(np.ascontiguousarray(image[lo:hi])).to("cuda") if hi > lo else torch.zeros(16, dtype=torch.uint8, device="cuda")
        ds.ds_unpack(self.plan, src.data_ptr(), lo, hi, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()

    def arena_host(self):
        return self.arena.cpu().numpy()

    def close(self):
        self.torch.cuda.synchronize()
        ds.ds_plan_destroy(self.plan)
        self.plan = None


def first_mismatch(a: np.ndarray, b: np.ndarray):
    if a.size != b.size:
        return f"sizes differ: {a.size} vs {b.size}"
    step = 1 << 26
    for lo in range(0, a.size, step):
        x, y = a[lo:lo + step], b[lo:lo + step]
        if not np.array_equal(x, y):
            i = int(np.flatnonzero(x != y)[0]) + lo
            n = int((x != y).sum())
            return f"first mismatch at byte {i} (got {a[i]:#x}, want {b[i]:#x}); {n}+ differing bytes in this window"
    return None
