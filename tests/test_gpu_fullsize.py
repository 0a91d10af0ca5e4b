"""GPU parity at the full sizes of the configurations, in the launch
configuration the benchmark times (default chunk size and kernel variant):
the whole image and the whole restored arena are compared with the CPU oracle
byte for byte (the oracle packs these sizes in seconds with host threads)."""
import os
import threading
import time

import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu

CASES = {
    "llama7b": (76, 1531543552),
    "fragmentation": (20000, None),
    "llama70b": (184, 7602667520),
}


@pytest.mark.parametrize("name", list(CASES))
def test_full_size_pack_and_restore(name):
    import paper_2601_16956_amd as ds
    from oracle import ds_oracle as orc
    import gpu_util as gu
    import torch

    n_shards, payload = CASES[name]
    cores = min(len(os.sched_getaffinity(0)), 16)
    t0 = time.time()
    w = W.by_name(name, workers=cores)
    print(f"[case] full size {name}: shards={len(w.shards)} payload={w.payload_bytes} arena={w.arena.size} "
          f"generated in {time.time() - t0:.1f}s", flush=True)
    assert len(w.shards) == n_shards
    if payload is not None:
        assert w.payload_bytes == payload
    n = len(w.shards)
    tab = orc.table(w.shards, w.arena.ctypes.data)
    total = orc.layout(tab, n, w.align)
    want = orc.pack(tab, n, total, threads=cores)
    print(f"[step] oracle image {total} bytes at {time.time() - t0:.1f}s", flush=True)

    dw = gu.DeviceWorkload(w)
    try:
        assert dw.total == total and dw.info["payload_bytes"] == w.payload_bytes
        assert dw.offsets == [int(tab[i].file_offset) for i in range(n)]
        image = torch.full((total,), 0xFF, dtype=torch.uint8, device="cuda")
        s = torch.cuda.current_stream().cuda_stream
        ds.ds_pack(dw.plan, image.data_ptr(), 0, total, s)
        torch.cuda.synchronize()
        got = image.cpu().numpy()
        print(f"[step] gpu image back at {time.time() - t0:.1f}s", flush=True)
        assert gu.first_mismatch(got, want) is None, gu.first_mismatch(got, want)
        del got
        # restore: wipe device memory, scatter the ORACLE's image, compare the whole arena
        dw.arena.fill_(0xA5)
        image.copy_(torch.from_numpy(want))
        ds.ds_unpack(dw.plan, image.data_ptr(), 0, total, s)
        torch.cuda.synchronize()
        back = dw.arena_host()
        w.arena[:] = 0xA5
        orc.unpack(tab, n, want)
        print(f"[step] restored arena back at {time.time() - t0:.1f}s", flush=True)
        assert gu.first_mismatch(back, w.arena) is None, gu.first_mismatch(back, w.arena)
        # the same image through the engine as the benchmark configures it (2 GiB ring of 128 MiB slots,
        # 2 x 2 GiB staging, one copy stream), with a consumer that copies every chunk out of the ring
        import ctypes
        del image                                                  # the tensors hold the oracle's image again
        eng = ds.ds_engine_create(2 << 30, 128 << 20, 2 << 30, 2, 0, 0, 1)
        try:
            ev = ds.ds_snapshot_async(eng, dw.plan, s)
            got = np.empty(total, dtype=np.uint8)
            seen = [0]

            def consumer():     # its own thread, as a flush would be: the gate below may block until it has made room
                while True:
                    ch = ds.ds_snapshot_next_chunk(ev)
                    if ch is None:
                        break
                    ptr, off, ln = ch
                    assert off == seen[0]
                    ctypes.memmove(got.ctypes.data + off, ptr, ln)
                    ds.ds_snapshot_release_chunk(ev, ptr)
                    seen[0] += ln

            th = threading.Thread(target=consumer)
            th.start()
            ds.ds_event_wait_on_stream(ev, s)
            th.join()
            seen = seen[0]
            ds.ds_event_wait(ev)
            st = ds.ds_event_stats(ev)
            ds.ds_event_destroy(ev)
            assert seen == total and st["n_pack_launches"] == (total + (2 << 30) - 1) // (2 << 30)
            print(f"[step] engine snapshot consumed at {time.time() - t0:.1f}s", flush=True)
            assert gu.first_mismatch(got, want) is None, gu.first_mismatch(got, want)
        finally:
            ds.ds_engine_destroy(eng)
    finally:
        dw.close()
