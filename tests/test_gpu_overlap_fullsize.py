"""The overlap configuration at its own size: snapshots of the Llama-7B rank's state taken every iteration
while the compute stream runs back-to-back 8192^3 bf16 GEMMs and a mutating update follows every gate
(DataStates-LLM Sec. V-A2: the next iteration starts right after the request, only the update phase waits;
Sec. IV-B: the state is immutable during forward/backward).  A consumer thread copies every chunk out of the
ring; every host image must equal the CPU oracle's image of the mirror state at that snapshot's request, so a
torn snapshot -- an update that overtook a gather, a ring slot or a piece of staging reused too early -- shows as
a mismatch.  Three engines: the benchmark's (ring 2 GiB of 128 MiB slots, staging 2 x 2 GiB, one copy stream),
a ring smaller than the image, and ring and staging both smaller than the image, which forces chunked
double-buffering on both sides."""
import ctypes
import os
import threading
import time

import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu

MiB, GiB = 1 << 20, 1 << 30
ITERS = 5
ENGINES = {
    # the benchmark's engine: one copy stream, 128 MiB ring slots
    "ring_2GiB_staging_2x2GiB": dict(ring=2 * GiB, chunk=128 * MiB, slot=2 * GiB, slots=2, streams=1),
    "ring_512MiB_staging_2x2GiB": dict(ring=512 * MiB, chunk=32 * MiB, slot=2 * GiB, slots=2, streams=2),
    "ring_512MiB_staging_1x512MiB": dict(ring=512 * MiB, chunk=128 * MiB, slot=512 * MiB, slots=1, streams=1),
}

_cache = {}


def _state():
    """The 7B rank and the oracle's images of it after 1..ITERS updates (made once for the three engines)."""
    if not _cache:
        from oracle import ds_oracle as orc
        cores = min(len(os.sched_getaffinity(0)), 16)
        t0 = time.time()
        w = W.by_name("llama7b", workers=cores)
        n = len(w.shards)
        arena0 = w.arena.copy()
        tab = orc.table(w.shards, w.arena.ctypes.data)
        total = orc.layout(tab, n, w.align)
        wants = np.empty((ITERS, total), dtype=np.uint8)
        for k in range(ITERS):
            w.arena += np.uint8(1)                       # the update, on the mirror: every byte + 1 (mod 256)
            orc.pack(tab, n, total, threads=cores, out=wants[k])
        print(f"[step] 7B rank and {ITERS} oracle images of {total} bytes in {time.time() - t0:.1f}s", flush=True)
        _cache.update(w=w, arena0=arena0, tab=tab, total=total, wants=wants, n=n, cores=cores)
    return _cache


@pytest.mark.parametrize("name", list(ENGINES))
def test_snapshots_under_the_gemm_stream_equal_the_oracle(name):
    import torch
    import paper_2601_16956_amd as ds
    from oracle import ds_oracle as orc
    import gpu_util as gu

    cfg = ENGINES[name]
    st = _state()
    w, total, wants, n = st["w"], st["total"], st["wants"], st["n"]
    print(f"[case] overlap at full size, engine {name}", flush=True)
    s = torch.cuda.current_stream().cuda_stream
    arena = torch.from_numpy(st["arena0"]).to("cuda")
    descs = ds.make_descs(w.shards, arena.data_ptr())
    assert ds.ds_layout_assign(descs, n, w.align) == total
    plan = ds.ds_plan_create(descs, n, w.align, ds.DS_PLAN_STRICT | ds.DS_PLAN_CHECK_MEMORY)
    eng = ds.ds_engine_create(cfg["ring"], cfg["chunk"], cfg["slot"], cfg["slots"], 0, 0, cfg["streams"])
    M = 8192
    A = torch.randn(M, M, device="cuda", dtype=torch.bfloat16)
    B = torch.randn(M, M, device="cuda", dtype=torch.bfloat16)
    C = torch.empty(M, M, device="cuda", dtype=torch.bfloat16)
    G = 32                                               # ~28 ms of GEMMs: about one snapshot's link time
    gots = np.empty((ITERS, total), dtype=np.uint8)
    events, errors = [], []
    have = threading.Condition()

    def consumer():                                      # one thread for all snapshots, in request order
        try:
            for k in range(ITERS):
                with have:
                    have.wait_for(lambda: len(events) > k or errors)
                    if errors:
                        return
                    ev = events[k]
                at = 0
                while True:
                    ch = ds.ds_snapshot_next_chunk(ev)
                    if ch is None:
                        break
                    ptr, off, ln = ch
                    assert off == at, (k, off, at)
                    ctypes.memmove(gots[k].ctypes.data + off, ptr, ln)
                    ds.ds_snapshot_release_chunk(ev, ptr)
                    at += ln
                assert at == total, (k, at)
        except BaseException as e:                       # noqa: BLE001 -- reported by the main thread
            errors.append(e)

    th = threading.Thread(target=consumer)
    th.start()
    try:
        prev = None
        t0 = time.time()
        for k in range(ITERS):
            for _ in range(G):                           # "forward/backward": the state is only read
                torch.matmul(A, B, out=C)
            if prev is not None:
                ds.ds_event_wait_on_stream(prev, s)      # the lazy gate
            arena.add_(1)                                # the mutating update phase, right behind the gate
            prev = ds.ds_snapshot_async(eng, plan, s)
            with have:
                events.append(prev)
                have.notify_all()
        ds.ds_event_wait_on_stream(prev, s)
        arena.add_(1)                                    # one more update behind the last gate: it must not show
        th.join()
        assert not errors, errors
        torch.cuda.synchronize()
        print(f"[step] {ITERS} iterations and their snapshots consumed in {time.time() - t0:.2f}s", flush=True)
        launches = []
        for ev in events:
            ds.ds_event_wait(ev)
            launches.append(ds.ds_event_stats(ev)["n_pack_launches"])
            ds.ds_event_destroy(ev)
        events.clear()
        assert launches == [-(-total // cfg["slot"])] * ITERS, launches
        for k in range(ITERS):
            bad = gu.first_mismatch(gots[k], wants[k])
            assert bad is None, (name, "snapshot", k, bad)
        print("[step] every image equals the oracle's", flush=True)
        # the state itself went through ITERS + 1 updates
        after = arena.cpu().numpy()
        assert np.array_equal(after, st["arena0"] + np.uint8(ITERS + 1))
        # restore of the last image (as captured by the engine) == the oracle's restore of its own image
        arena.fill_(0xA5)
        image = torch.from_numpy(gots[ITERS - 1]).to("cuda")
        ds.ds_unpack(plan, image.data_ptr(), 0, total, s)
        torch.cuda.synchronize()
        back = arena.cpu().numpy()
        keep = w.arena.copy()
        try:
            w.arena[:] = 0xA5
            orc.unpack(st["tab"], n, wants[ITERS - 1])
            bad = gu.first_mismatch(back, w.arena)
        finally:
            w.arena[:] = keep
        assert bad is None, (name, "restore", bad)
    finally:
        if th.is_alive():
            with have:
                errors.append(RuntimeError("main thread failed"))
                have.notify_all()
            th.join(timeout=30)
        torch.cuda.synchronize()
        for ev in events:
            ds.ds_event_destroy(ev)
        ds.ds_engine_destroy(eng)
        ds.ds_plan_destroy(plan)
