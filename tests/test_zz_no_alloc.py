"""ds_pack_noalloc (the gather whose tables live in a static device array) against ds_pack, through the
C ABI, byte for byte: two calls in a row on one stream, the second with a smaller input, so the array still
holds the first call's tables when the second one arrives; then ranges, a third call that is larger again,
and the size limit."""
import ctypes

import numpy as np
import pytest

import workloads as W
from workloads.configs import Shard, Workload

pytestmark = pytest.mark.gpu


def _image(ds, torch, fn, plan, lo, hi):
    out = torch.full((max(hi - lo, 16),), 0xFF, dtype=torch.uint8, device="cuda")
    fn(plan, out.data_ptr(), lo, hi, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    return out[:hi - lo].cpu().numpy()


def test_no_alloc_gather_equals_ds_pack_on_two_calls_in_a_row():
    import torch
    import paper_2601_16956_amd as ds
    import gpu_util as gu

    cases = [("tiny_gpt", W.tiny_gpt()),                                                  # 26.7 MB, 118 shards
             ("frag_small", W.fragmentation(700, max_bytes=1 << 15, seed=77)),            # smaller: a few MB
             ("frag_larger_again", W.fragmentation(3000, max_bytes=1 << 16, seed=78))]
    sizes = []
    for name, w in cases:
        print(f"[case] no-alloc gather {name} shards={len(w.shards)} payload={w.payload_bytes}", flush=True)
        want, offs, _ = gu.oracle_image(w)
        dw = gu.DeviceWorkload(w)                       # device plan: what ds_pack uses
        # the same table as a host-only plan: creating it touches no device
        hd = ds.make_descs(w.shards, dw.arena.data_ptr())
        assert ds.ds_layout_assign(hd, dw.n, w.align) == dw.total
        hplan = ds.ds_plan_create(hd, dw.n, w.align, ds.DS_PLAN_HOST_ONLY)
        try:
            ref = _image(ds, torch, ds.ds_pack, dw.plan, 0, dw.total)
            assert gu.first_mismatch(ref, want) is None
            got = _image(ds, torch, ds.ds_pack_noalloc, hplan, 0, dw.total)
            assert gu.first_mismatch(got, ref) is None, (name, gu.first_mismatch(got, ref))
            # a device plan serves as well (its host tables are the same)
            got = _image(ds, torch, ds.ds_pack_noalloc, dw.plan, 0, dw.total)
            assert gu.first_mismatch(got, ref) is None, (name, "device plan", gu.first_mismatch(got, ref))
            # ranges that cut chunks at both ends
            for lo, hi in ((16, dw.total - 16), (48 * 1024 + 16, 112 * 1024 + 32), (dw.total - 4096, dw.total)):
                lo, hi = max(0, lo) & ~15, min(dw.total, hi) & ~15
                if lo >= hi:
                    continue
                part = _image(ds, torch, ds.ds_pack_noalloc, hplan, lo, hi)
                assert gu.first_mismatch(part, ref[lo:hi]) is None, (name, lo, hi)
            ds.ds_pack_noalloc(hplan, 0, 64, 64, 0)       # empty range: nothing to do, no pointer needed
            sizes.append(dw.total)
        finally:
            ds.ds_plan_destroy(hplan)
            dw.close()
    assert sizes[1] < sizes[0] and sizes[2] > sizes[1]


def test_no_alloc_gather_refuses_tables_beyond_its_static_memory():
    import torch
    import paper_2601_16956_amd as ds

    # 4 GiB as one contiguous tensor: 262 144 chunks x 36 bytes of tables > 4 MiB.  A host-only plan of a
    # tensor that does not exist; the call must refuse before it enqueues or touches anything.
    arena = np.zeros(16, dtype=np.uint8)
    sh = [Shard("huge", "u8", (1 << 32,), (1,), 0, 1)]
    d = ds.make_descs(sh, 1 << 40)
    total = ds.ds_layout_assign(d, 1, 4096)
    plan = ds.ds_plan_create(d, 1, 4096, ds.DS_PLAN_HOST_ONLY)
    try:
        assert ds.ds_plan_info(plan)["n_chunks"] * 36 > ds.DS_PACK_NOALLOC_TABLE_BYTES
        dst = torch.zeros(4096, dtype=torch.uint8, device="cuda")
        with pytest.raises(ds.DsError) as e:
            ds.ds_pack_noalloc(plan, dst.data_ptr(), 0, 4096, torch.cuda.current_stream().cuda_stream)
        assert e.value.code == ds.DS_ETOOBIG
        with pytest.raises(ds.DsError) as e:
            ds.ds_pack_noalloc(plan, dst.data_ptr(), 0, total + 16, 0)
        assert e.value.code == ds.DS_ERANGE
        torch.cuda.synchronize()
        assert int(dst.sum().item()) == 0
    finally:
        ds.ds_plan_destroy(plan)
    del arena
