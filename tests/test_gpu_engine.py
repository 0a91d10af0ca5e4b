"""GPU tests of the snapshot engine (request -> gather -> chunked copies into
the pinned ring -> consumer), against the CPU oracle byte for byte."""
import ctypes
import threading
import time

import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu

MiB = 1 << 20


def _mods():
    import paper_2601_16956_amd as ds
    from oracle import ds_oracle as orc
    import gpu_util
    import torch
    return ds, orc, gpu_util, torch


def _drain(ds, ev, total, delay=0.0, hold=1):
    """Consumer: copies every chunk out of the ring into a host image.  `hold`
    chunks are kept unreleased at a time (1 = release at once)."""
    img = np.empty(total, dtype=np.uint8)
    held = []
    seen = 0
    while True:
        got = ds.ds_snapshot_next_chunk(ev)
        if got is None:
            break
        ptr, off, ln = got
        assert off == seen, "chunks must come in file order"
        img[off:off + ln] = np.ctypeslib.as_array((ctypes.c_uint8 * ln).from_address(ptr))
        seen += ln
        held.append(ptr)
        if delay:
            time.sleep(delay)
        while len(held) >= hold:
            ds.ds_snapshot_release_chunk(ev, held.pop(0))
    for p in held:
        ds.ds_snapshot_release_chunk(ev, p)
    assert seen == total
    return img


@pytest.mark.parametrize("cfg", [
    dict(ring=4 * MiB, chunk=1 * MiB, slot=4 * MiB, slots=2, copy_streams=1),
    dict(ring=2 * MiB, chunk=1 * MiB, slot=1 * MiB, slots=1, copy_streams=1),
    dict(ring=8 * MiB, chunk=2 * MiB, slot=8 * MiB, slots=3, copy_streams=2),
    dict(ring=64 * MiB, chunk=32 * MiB, slot=64 * MiB, slots=1, copy_streams=1),   # image fits one slot
    dict(ring=8 * MiB, chunk=1 * MiB, slot=8 * MiB, slots=2, copy_streams=1, first=1 * MiB),  # short first launch
    dict(ring=8 * MiB, chunk=2 * MiB, slot=8 * MiB, slots=2, copy_streams=1, grid=64),        # grid-limited gather
])
def test_snapshot_with_consumer_matches_oracle(cfg):
    ds, orc, gu, torch = _mods()
    w = W.tiny_gpt()
    print(f"[case] snapshot consumer {cfg}", flush=True)
    want, _, _ = gu.oracle_image(w)
    dw = gu.DeviceWorkload(w)
    eng = ds.ds_engine_create(cfg["ring"], cfg["chunk"], cfg["slot"], cfg["slots"], cfg.get("grid", 0), 0, cfg["copy_streams"],
                              cfg.get("first", 0))
    try:
        for rep in range(2):                                  # the second run reuses ring, staging, events
            ev = ds.ds_snapshot_async(eng, dw.plan, torch.cuda.current_stream().cuda_stream)
            got = _drain(ds, ev, dw.total, hold=1 + rep)
            ds.ds_event_wait(ev)
            assert ds.ds_event_query(ev) == ds.DS_OK
            st = ds.ds_event_stats(ev)
            assert st["image_bytes"] == dw.total and st["n_copies"] == -(-dw.total // cfg["chunk"])
            assert st["n_pack_launches"] >= 1 and st["total_ms"] >= st["capture_ms"] > 0
            ds.ds_event_destroy(ev)
            assert gu.first_mismatch(got, want) is None, gu.first_mismatch(got, want)
    finally:
        ds.ds_engine_destroy(eng)
        dw.close()


def test_gate_keeps_the_snapshot_consistent_while_state_mutates():
    """Sec. V-A2: the next iteration starts right after the request; the update
    phase is gated.  Here the 'update' adds 1 to every byte of device memory,
    enqueued directly behind the gate, with no host synchronisation; every
    snapshot must still show the state at its own request."""
    ds, orc, gu, torch = _mods()
    w = W.fragmentation(1500, max_bytes=1 << 18, seed=31)
    dw = gu.DeviceWorkload(w)
    eng = ds.ds_engine_create(16 * MiB, 4 * MiB, 16 * MiB, 2, 0, 0, 1)
    s = torch.cuda.current_stream().cuda_stream
    busy = torch.randn(2048, 2048, device="cuda")
    try:
        events, wants = [], []
        mirror = w.arena.copy()
        for it in range(3):
            print(f"[case] gate iteration {it}", flush=True)
            w.arena[:] = mirror
            wants.append(gu.oracle_image(w)[0].copy())
            ev = ds.ds_snapshot_async(eng, dw.plan, s)
            for _ in range(4):                                 # "forward/backward": state is only read
                busy = busy @ busy * 1e-3
            # consumer runs concurrently so that ring slots come back
            box = {}
            th = threading.Thread(target=lambda: box.setdefault("img", _drain(ds, ev, dw.total)))
            th.start()
            ds.ds_event_wait_on_stream(ev, s)                  # the lazy gate
            dw.arena.add_(1)                                   # the mutating "update"
            mirror = mirror + np.uint8(1)
            th.join()
            events.append((ev, box["img"]))
        torch.cuda.synchronize()
        for it, ((ev, got), want) in enumerate(zip(events, wants)):
            ds.ds_event_wait(ev)
            assert gu.first_mismatch(got, want) is None, (it, gu.first_mismatch(got, want))
            ds.ds_event_destroy(ev)
        assert np.array_equal(dw.arena_host(), mirror)
    finally:
        ds.ds_engine_destroy(eng)
        dw.close()


def test_back_pressure_slow_consumer_and_queued_snapshots():
    """Sec. V-A2 last paragraph: with the ring full the next request waits for
    eviction.  Two snapshots are requested back to back on a 2-slot ring; the
    consumer is slow; nothing is lost or torn."""
    ds, orc, gu, torch = _mods()
    w = W.tiny_gpt()
    want, _, _ = gu.oracle_image(w)
    dw = gu.DeviceWorkload(w)
    eng = ds.ds_engine_create(2 * MiB, 1 * MiB, 2 * MiB, 2, 0, 0, 2)
    s = torch.cuda.current_stream().cuda_stream
    try:
        ev1 = ds.ds_snapshot_async(eng, dw.plan, s)
        ev2 = ds.ds_snapshot_async(eng, dw.plan, s)
        time.sleep(0.2)
        # the ring holds 2 of ~26 chunks: neither snapshot can be complete yet
        assert ds.ds_event_query(ev1) == ds.DS_NOT_READY
        assert ds.ds_event_query(ev2) == ds.DS_NOT_READY
        print("[case] back-pressure drain 1", flush=True)
        got1 = _drain(ds, ev1, dw.total, delay=0.002)
        print("[case] back-pressure drain 2", flush=True)
        got2 = _drain(ds, ev2, dw.total)
        ds.ds_event_wait(ev1)
        ds.ds_event_wait(ev2)
        assert gu.first_mismatch(got1, want) is None
        assert gu.first_mismatch(got2, want) is None
        ds.ds_event_destroy(ev1)
        ds.ds_event_destroy(ev2)
    finally:
        ds.ds_engine_destroy(eng)
        dw.close()


def test_gates_of_queued_snapshots_do_not_wait_for_the_host_ring():
    """Staging holds three images, the host ring two chunks, and nobody consumes:
    the copies of the first snapshot are stuck behind the full ring, yet the
    gathers of all three are issued ahead, so every gate opens and the state may
    be mutated between the requests.  Drained afterwards, each snapshot shows
    the state at its own request."""
    ds, orc, gu, torch = _mods()
    w = W.tiny_gpt()
    dw = gu.DeviceWorkload(w)
    assert 3 * dw.total <= 96 * MiB
    eng = ds.ds_engine_create(2 * MiB, 1 * MiB, 32 * MiB, 3, 0, 0, 2)
    s = torch.cuda.current_stream().cuda_stream
    try:
        mirror = w.arena.copy()
        events, wants = [], []
        for it in range(3):
            print(f"[case] queued gate {it}", flush=True)
            w.arena[:] = mirror
            wants.append(gu.oracle_image(w)[0].copy())
            ev = ds.ds_snapshot_async(eng, dw.plan, s)
            ds.ds_event_wait_on_stream(ev, s)                  # must not block: no consumer is running
            dw.arena.add_(1)
            mirror = mirror + np.uint8(1)
            events.append(ev)
        ds.ds_event_wait_captured(events[-1])                  # every source byte of all three is in staging
        for ev in events:
            assert ds.ds_event_query(ev) == ds.DS_NOT_READY    # 2 ring slots of ~26 chunks: none can be complete
        for it, (ev, want) in enumerate(zip(events, wants)):
            got = _drain(ds, ev, dw.total)
            ds.ds_event_wait(ev)
            assert gu.first_mismatch(got, want) is None, (it, gu.first_mismatch(got, want))
            ds.ds_event_destroy(ev)
        assert np.array_equal(dw.arena_host(), mirror)
    finally:
        ds.ds_engine_destroy(eng)
        dw.close()


@pytest.mark.parametrize("cfg", [
    dict(ring=3 * MiB, chunk=1 * MiB, slot=2 * MiB, slots=3, copy_streams=2),
    dict(ring=8 * MiB, chunk=2 * MiB, slot=8 * MiB, slots=2, copy_streams=2, first=2 * MiB),
    dict(ring=2 * MiB, chunk=1 * MiB, slot=1 * MiB, slots=1, copy_streams=1),
])
def test_random_sequence_of_snapshots_of_three_plans(cfg):
    """Three shard sets of very different sizes share one engine whose staging
    is smaller than the largest image: ten snapshots in random order, each gated
    and followed by an update of its own tensors, drained by one consumer
    thread in request order.  Every image must be the oracle's image of the
    state at its request (pieces of staging are handed from snapshot to
    snapshot, wrap around, and wait for the ring)."""
    import queue
    ds, orc, gu, torch = _mods()
    sets = [W.tiny_gpt(), W.fragmentation(400, max_bytes=1 << 16, seed=5), W.fragmentation(12, max_bytes=1 << 12, seed=6)]
    dws = [gu.DeviceWorkload(w) for w in sets]
    mirrors = [w.arena.copy() for w in sets]
    eng = ds.ds_engine_create(cfg["ring"], cfg["chunk"], cfg["slot"], cfg["slots"], 0, 0, cfg["copy_streams"],
                              cfg.get("first", 0))
    s = torch.cuda.current_stream().cuda_stream
    todo, results = queue.Queue(), []

    def consumer():
        while True:
            item = todo.get()
            if item is None:
                return
            ev, total = item
            results.append(_drain(ds, ev, total))

    th = threading.Thread(target=consumer)
    th.start()
    rng = np.random.default_rng(2601)
    wants, events = [], []
    try:
        for it in range(10):
            p = int(rng.integers(0, 3))
            print(f"[case] random sequence {cfg} step {it} plan {p}", flush=True)
            sets[p].arena[:] = mirrors[p]
            wants.append(gu.oracle_image(sets[p])[0].copy())
            ev = ds.ds_snapshot_async(eng, dws[p].plan, s)
            todo.put((ev, dws[p].total))
            ds.ds_event_wait_on_stream(ev, s)                  # the consumer is another thread: this may wait for it
            dws[p].arena.add_(it + 1)
            mirrors[p] = mirrors[p] + np.uint8(it + 1)
            events.append(ev)
        todo.put(None)
        th.join()
        torch.cuda.synchronize()
        for it, (ev, got, want) in enumerate(zip(events, results, wants)):
            ds.ds_event_wait(ev)
            assert gu.first_mismatch(got, want) is None, (it, gu.first_mismatch(got, want))
            ds.ds_event_destroy(ev)
        for p in range(3):
            assert np.array_equal(dws[p].arena_host(), mirrors[p])
    finally:
        if th.is_alive():
            todo.put(None)
            th.join()
        ds.ds_engine_destroy(eng)
        for dw in dws:
            dw.close()


def test_auto_release_and_state_errors():
    ds, orc, gu, torch = _mods()
    w = W.tiny_gpt()
    dw = gu.DeviceWorkload(w)
    s = torch.cuda.current_stream().cuda_stream
    eng = ds.ds_engine_create(4 * MiB, 1 * MiB, 4 * MiB, 2, 0, ds.DS_ENGINE_AUTO_RELEASE, 1)
    try:
        print("[case] auto release", flush=True)
        ev = ds.ds_snapshot_async(eng, dw.plan, s)
        with pytest.raises(ds.DsError) as e:
            ds.ds_snapshot_next_chunk(ev)
        assert e.value.code == ds.DS_ESTATE
        with pytest.raises(ds.DsError) as e:
            ds.ds_engine_destroy(eng)                          # an event is still alive
        assert e.value.code == ds.DS_EBUSY
        ds.ds_event_wait_captured(ev)
        ds.ds_event_wait(ev)
        st = ds.ds_event_stats(ev)
        assert st["payload_bytes"] == w.payload_bytes and st["pack_ms"] > 0 and st["copy_ms"] > 0
        ds.ds_event_destroy(ev)
    finally:
        ds.ds_engine_destroy(eng)
    eng = ds.ds_engine_create(4 * MiB, 1 * MiB, 4 * MiB, 2, 0, 0, 1)
    try:
        print("[case] destroy drains an unconsumed snapshot", flush=True)
        ev = ds.ds_snapshot_async(eng, dw.plan, s)
        got = ds.ds_snapshot_next_chunk(ev)
        with pytest.raises(ds.DsError) as e:
            ds.ds_snapshot_release_chunk(ev, got[0] + 4096)    # not a slot address
        assert e.value.code == ds.DS_ESTATE
        ds.ds_event_destroy(ev)                                # gives back what is held, drains the rest
    finally:
        ds.ds_engine_destroy(eng)
        dw.close()
    for bad in [dict(d2h_chunk_bytes=1000), dict(d2h_chunk_bytes=MiB, stage_slot_bytes=MiB + 4096),
                dict(host_ring_bytes=MiB, d2h_chunk_bytes=2 * MiB), dict(copy_streams=3),
                dict(d2h_chunk_bytes=MiB, stage_slot_bytes=4 * MiB, first_launch_bytes=8 * MiB)]:
        with pytest.raises(ds.DsError) as e:
            ds.ds_engine_create(**bad)
        assert e.value.code == ds.DS_EINVAL


@pytest.mark.parametrize("cfg", [
    dict(ring=4 * MiB, chunk=1 * MiB, slot=4 * MiB, slots=2, ahead=1),
    dict(ring=2 * MiB, chunk=1 * MiB, slot=1 * MiB, slots=1, ahead=2),
    dict(ring=8 * MiB, chunk=2 * MiB, slot=8 * MiB, slots=3, ahead=3),
    dict(ring=64 * MiB, chunk=32 * MiB, slot=64 * MiB, slots=1, ahead=1),
])
def test_restore_pipeline_matches_oracle(cfg):
    """Host image -> ring slots -> staging -> scatter; the whole arena (wiped to
    0xA5 first) is compared with the oracle's unpack into a wiped host arena."""
    ds, orc, gu, torch = _mods()
    w = W.fragmentation(1200, max_bytes=1 << 16, seed=71)
    print(f"[case] restore {cfg}", flush=True)
    img, offs, tab = gu.oracle_image(w)
    dw = gu.DeviceWorkload(w, arena_fill=0xA5)
    eng = ds.ds_engine_create(cfg["ring"], cfg["chunk"], cfg["slot"], cfg["slots"], 0, 0, 1)
    s = torch.cuda.current_stream().cuda_stream
    try:
        for rep in range(2):
            dw.arena.fill_(0xA5)
            ev = ds.ds_restore_begin(eng, dw.plan, s)
            with pytest.raises(ds.DsError) as e:                  # one event at a time on a restoring engine
                ds.ds_restore_begin(eng, dw.plan, s)
            assert e.value.code == ds.DS_EBUSY
            held = []
            while True:
                got = ds.ds_restore_next_slot(ev)
                if got is not None:
                    ptr, off, ln = got
                    ctypes.memmove(ptr, img[off:off + ln].ctypes.data, ln)
                    held.append(ptr)
                while held and (got is None or len(held) >= cfg["ahead"]):
                    ds.ds_restore_submit(ev, held.pop(0))
                if got is None:
                    break
            ds.ds_event_wait_on_stream(ev, s)
            probe = dw.arena.clone()                              # on the gated stream: sees the restored state
            ds.ds_event_wait(ev)
            assert ds.ds_event_query(ev) == ds.DS_OK
            st = ds.ds_event_stats(ev)
            assert st["n_pack_launches"] >= 1 and st["total_ms"] > 0
            ds.ds_event_destroy(ev)
            back = dw.arena_host()
            if rep == 0:
                w.arena[:] = 0xA5
                orc.unpack(tab, len(w.shards), img)
            assert gu.first_mismatch(back, w.arena) is None, gu.first_mismatch(back, w.arena)
            assert gu.first_mismatch(probe.cpu().numpy(), w.arena) is None
    finally:
        ds.ds_engine_destroy(eng)
        dw.close()


def test_restore_state_errors():
    ds, orc, gu, torch = _mods()
    w = W.tiny_gpt()
    dw = gu.DeviceWorkload(w)
    eng = ds.ds_engine_create(2 * MiB, 1 * MiB, 2 * MiB, 2, 0, 0, 1)
    s = torch.cuda.current_stream().cuda_stream
    try:
        ev = ds.ds_restore_begin(eng, dw.plan, s)
        a = ds.ds_restore_next_slot(ev)
        b = ds.ds_restore_next_slot(ev)
        with pytest.raises(ds.DsError) as e:                      # both slots are with the caller
            ds.ds_restore_next_slot(ev)
        assert e.value.code == ds.DS_EBUSY
        with pytest.raises(ds.DsError) as e:                      # out of order
            ds.ds_restore_submit(ev, b[0])
        assert e.value.code == ds.DS_ESTATE
        with pytest.raises(ds.DsError) as e:                      # not finished: nothing to wait for yet
            ds.ds_event_wait(ev)
        assert e.value.code == ds.DS_ESTATE
        with pytest.raises(ds.DsError) as e:
            ds.ds_snapshot_next_chunk(ev)
        assert e.value.code == ds.DS_ESTATE
        with pytest.raises(ds.DsError) as e:                      # ring and staging belong to the restore
            ds.ds_snapshot_async(eng, dw.plan, s)
        assert e.value.code == ds.DS_EBUSY
        ds.ds_restore_submit(ev, a[0])
        ds.ds_event_destroy(ev)                                   # abandoning a restore is allowed
        ev = ds.ds_snapshot_async(eng, dw.plan, s)                # the engine is usable again
        with pytest.raises(ds.DsError) as e:
            ds.ds_restore_begin(eng, dw.plan, s)
        assert e.value.code == ds.DS_EBUSY
        with pytest.raises(ds.DsError) as e:
            ds.ds_restore_next_slot(ev)
        assert e.value.code == ds.DS_ESTATE
        ds.ds_event_destroy(ev)
    finally:
        ds.ds_engine_destroy(eng)
        dw.close()


@pytest.mark.parametrize("flags_name", ["buffered", "direct_sync", "uring", "uring_direct"])
def test_flush_to_file_and_restore_from_file(tmp_path, flags_name):
    """GPU -> ring -> file with background writer threads, then file -> ring ->
    GPU; the file must be the oracle's image, the restored arena the oracle's
    unpack of it."""
    ds, orc, gu, torch = _mods()
    flags = {"buffered": 0, "direct_sync": ds.DS_FILE_DIRECT | ds.DS_FILE_SYNC, "uring": ds.DS_FILE_URING,
             "uring_direct": ds.DS_FILE_URING | ds.DS_FILE_DIRECT}[flags_name]
    if flags & ds.DS_FILE_URING:
        print(f"[info] io_uring available: {ds.ds_config_get('io_uring_available')}", flush=True)
    w = W.fragmentation(2500, max_bytes=1 << 17, seed=91)
    print(f"[case] file tier {flags_name}", flush=True)
    want, offs, tab = gu.oracle_image(w)
    dw = gu.DeviceWorkload(w)
    eng = ds.ds_engine_create(6 * MiB, 1 * MiB, 8 * MiB, 2, 0, 0, 2)     # ring far smaller than the image
    s = torch.cuda.current_stream().cuda_stream
    path = str(tmp_path / "image.bin")
    try:
        ev = ds.ds_snapshot_async(eng, dw.plan, s)
        fl = ds.ds_flush_start(ev, path, 3, flags)
        ds.ds_event_wait_on_stream(ev, s)
        nbytes, secs = ds.ds_flush_wait(fl)
        ds.ds_event_wait(ev)
        ds.ds_event_destroy(ev)
        assert nbytes == dw.total and secs > 0
        on_disk = np.fromfile(path, dtype=np.uint8)
        assert gu.first_mismatch(on_disk, want) is None, gu.first_mismatch(on_disk, want)

        dw.arena.fill_(0xA5)
        rev = ds.ds_restore_from_file(eng, dw.plan, path, 3, flags & ds.DS_FILE_DIRECT, s)
        ds.ds_event_wait(rev)
        ds.ds_event_destroy(rev)
        w.arena[:] = 0xA5
        orc.unpack(tab, len(w.shards), want)
        assert gu.first_mismatch(dw.arena_host(), w.arena) is None

        with pytest.raises(ds.DsError) as e:                       # a file that is too short
            with open(path, "r+b") as f:
                f.truncate(dw.total // 2)
            ds.ds_restore_from_file(eng, dw.plan, path, 2, 0, s)
        assert e.value.code == ds.DS_EIO
        with pytest.raises(ds.DsError) as e:
            ds.ds_restore_from_file(eng, dw.plan, str(tmp_path / "missing.bin"), 2, 0, s)
        assert e.value.code == ds.DS_EIO and ds.ds_last_errno() == 2
    finally:
        ds.ds_engine_destroy(eng)
        dw.close()


def test_checkpoint_file_from_a_snapshot_with_concurrent_object_log(tmp_path):
    """Snapshot -> ring -> tensor region of a checkpoint file while three
    threads append object chunks to the log behind it; the oracle's parser must
    find the oracle's image, every object and the plan's manifest; the file
    restores the tensors through the pipeline; a file of another plan is refused."""
    import threading
    from oracle import ckpt_format as fmt
    ds, orc, gu, torch = _mods()
    w = W.fragmentation(2500, max_bytes=1 << 17, seed=93)
    print("[case] checkpoint file", flush=True)
    want, offs, tab = gu.oracle_image(w)
    dw = gu.DeviceWorkload(w)
    eng = ds.ds_engine_create(6 * MiB, 1 * MiB, 8 * MiB, 2, 0, 0, 0)
    s = torch.cuda.current_stream().cuda_stream
    path = str(tmp_path / "rank0.ckpt")
    sent = {}

    def producer(t, ck):
        rng = np.random.default_rng(500 + t)
        mine = b""
        for k in range(40):
            data = rng.integers(0, 256, size=int(rng.choice([0, 7, 64, 5000])), dtype=np.uint8).tobytes()
            ds.ds_ckpt_append(ck, 70 + t, data)
            mine += data
        sent[70 + t] = mine

    try:
        ev = ds.ds_snapshot_async(eng, dw.plan, s)
        ck = ds.ds_ckpt_create(path, dw.plan, 0)
        ds.ds_ckpt_flush_snapshot(ck, ev, 3)
        with pytest.raises(ds.DsError) as e:
            ds.ds_ckpt_flush_snapshot(ck, ev, 3)
        assert e.value.code == ds.DS_ESTATE
        ts = [threading.Thread(target=producer, args=(t, ck)) for t in range(3)]
        for t in ts:
            t.start()
        ds.ds_event_wait_on_stream(ev, s)
        for t in ts:
            t.join()
        nbytes, secs = ds.ds_ckpt_finish(ck)
        ds.ds_event_wait(ev)
        ds.ds_event_destroy(ev)
        blob = open(path, "rb").read()
        assert nbytes == len(blob)
        back = fmt.parse_file(blob)
        assert gu.first_mismatch(np.frombuffer(back["image"], dtype=np.uint8), want) is None
        assert back["objects"] == sent
        n = len(w.shards)
        assert back["tensors"] == [ds.ds_plan_shard(dw.plan, i)[:2] + (ds.ds_plan_shard_shape(dw.plan, i),)
                                   + ds.ds_plan_shard(dw.plan, i)[2:] for i in range(n)]

        r = ds.ds_ckpt_open(path)
        dw.arena.fill_(0xA5)
        rev = ds.ds_ckpt_restore(r, eng, dw.plan, 3, 0, s)
        ds.ds_event_wait(rev)
        ds.ds_event_destroy(rev)
        w.arena[:] = 0xA5
        orc.unpack(tab, n, want)
        assert gu.first_mismatch(dw.arena_host(), w.arena) is None
        for oid, data in sent.items():
            assert ds.ds_ckpt_object_read(r, oid) == data
        # a plan over other shards does not match this file
        w2 = W.tiny_gpt()
        dw2 = gu.DeviceWorkload(w2)
        with pytest.raises(ds.DsError) as e:
            ds.ds_ckpt_restore(r, eng, dw2.plan, 2, 0, s)
        assert e.value.code == ds.DS_EFORMAT
        dw2.close()
        ds.ds_ckpt_close(r)
    finally:
        ds.ds_engine_destroy(eng)
        dw.close()


def test_rank_checkpoint_split_over_several_files(tmp_path):
    """A rank that writes several files per checkpoint (Sec. VI-D: 20 for the 7B
    rank) uses one plan and one checkpoint writer per file, all through one
    engine and in flight together.  Every file must hold the oracle's image of its
    own shards, and restoring the files one after the other must bring back
    every tensor."""
    from oracle import ckpt_format as fmt
    ds, orc, gu, torch = _mods()
    w = W.fragmentation(900, max_bytes=1 << 18, seed=41)
    n = len(w.shards)
    print("[case] several files", flush=True)
    arena = torch.from_numpy(w.arena).to("cuda")
    cuts = [0, n // 7, n // 3, n // 3 + 1, (3 * n) // 4, n]           # five files, one of them a single shard
    eng = ds.ds_engine_create(4 * MiB, 1 * MiB, 2 * MiB, 2, 0, 0, 0)  # ring smaller than the sum of the images
    s = torch.cuda.current_stream().cuda_stream
    files = []
    try:
        for k, (a, b) in enumerate(zip(cuts[:-1], cuts[1:])):
            shards = w.shards[a:b]
            descs = ds.make_descs(shards, arena.data_ptr())
            total = ds.ds_layout_assign(descs, b - a, w.align)
            plan = ds.ds_plan_create(descs, b - a, w.align, ds.DS_PLAN_STRICT)
            tab = orc.table(shards, w.arena.ctypes.data)
            assert orc.layout(tab, b - a, w.align) == total
            files.append({"plan": plan, "tab": tab, "n": b - a, "total": total,
                          "want": orc.pack(tab, b - a, total, threads=4), "path": str(tmp_path / f"rank0_{k}.ckpt")})
        for f in files:
            f["ev"] = ds.ds_snapshot_async(eng, f["plan"], s)
            f["ck"] = ds.ds_ckpt_create(f["path"], f["plan"], ds.DS_FILE_DIRECT)
            ds.ds_ckpt_flush_snapshot(f["ck"], f["ev"], 2)
            ds.ds_ckpt_append(f["ck"], 1, b"file %d" % len(f["path"]))
        ds.ds_event_wait_on_stream(files[-1]["ev"], s)                 # snapshots run in order: this gate covers all
        arena.fill_(0xA5)                                              # the update phase may now overwrite everything
        torch.cuda.synchronize()
        for f in files:
            ds.ds_ckpt_finish(f["ck"])
            ds.ds_event_wait(f["ev"])
            ds.ds_event_destroy(f["ev"])
            back = fmt.parse_file(open(f["path"], "rb").read())
            assert gu.first_mismatch(np.frombuffer(back["image"], dtype=np.uint8), f["want"]) is None, f["path"]
            assert back["objects"] == {1: b"file %d" % len(f["path"])}
        mirror = w.arena.copy()
        w.arena[:] = 0xA5
        for f in files:
            r = ds.ds_ckpt_open(f["path"])
            rev = ds.ds_ckpt_restore(r, eng, f["plan"], 2, ds.DS_FILE_DIRECT, s)
            ds.ds_event_wait(rev)
            ds.ds_event_destroy(rev)
            ds.ds_ckpt_close(r)
            orc.unpack(f["tab"], f["n"], f["want"])
        assert gu.first_mismatch(arena.cpu().numpy(), w.arena) is None
        # every addressed byte is back (the rest of the arena keeps the 0xA5 written above)
        for f in files:
            got = orc.pack(f["tab"], f["n"], f["total"], threads=4)
            assert gu.first_mismatch(got, f["want"]) is None
        w.arena[:] = mirror
    finally:
        ds.ds_engine_destroy(eng)
        torch.cuda.synchronize()
        for f in files:
            ds.ds_plan_destroy(f["plan"])


@pytest.mark.parametrize("fflags", ["direct", "uring", "buffered"])
def test_rank_checkpoint_of_several_files_through_one_plan(tmp_path, fflags):
    """The same rank with ONE plan over all its files (Sec. VI-D; Sec. V-A3: one composite provider lays
    out everything the rank owns): one gather launch sequence and one snapshot cover all files, the
    flush cuts the ring's chunks at the files' boundaries.  The plan's image must be the oracle's
    per-file images one behind the other, every file must be the oracle's file of its own shards, and
    ONE restore out of all files must bring back every tensor.  The ring is smaller than the image
    and its chunks are not aligned with the files, so chunks span two and more files."""
    from oracle import ckpt_format as fmt
    ds, orc, gu, torch = _mods()
    file_flags = {"direct": ds.DS_FILE_DIRECT, "uring": ds.DS_FILE_URING | ds.DS_FILE_DIRECT, "buffered": 0}[fflags]
    w = W.fragmentation(900, max_bytes=1 << 18, seed=41)
    n = len(w.shards)
    print(f"[case] several files through one plan, {fflags}", flush=True)
    arena = torch.from_numpy(w.arena).to("cuda")
    # seven files: one of a single shard, one empty, and a run of small shards dealt out in turn over two files
    # (so that neighbours in the table land in different files)
    cuts = [0, n // 7, n // 3, n // 3 + 1, (3 * n) // 4, n]
    file_of = []
    for i in range(n):
        f = next(k for k in range(5) if cuts[k] <= i < cuts[k + 1])
        file_of.append(f if f < 4 else 5 + (i & 1))                   # files 0..3, 5, 6; file 4 stays empty
    n_files = 7
    sizes = [sh.nbytes for sh in w.shards]
    offs, regions, begins = fmt.rank_files(sizes, file_of, n_files, w.align)
    alone, tabs = [], []
    for f in range(n_files):
        sub = [sh for sh, g in zip(w.shards, file_of) if g == f]
        t = orc.table(sub, w.arena.ctypes.data)
        assert orc.layout(t, len(sub), w.align) == regions[f]
        alone.append(orc.pack(t, len(sub), regions[f], threads=4))
        tabs.append((t, len(sub)))
    want_image = np.concatenate(alone)
    descs = ds.make_descs(w.shards, arena.data_ptr())
    got_regions, total = ds.ds_layout_assign_files(descs, file_of, n, n_files, w.align)
    assert got_regions == regions and total == want_image.size
    plan = ds.ds_plan_create_files(descs, file_of, n, n_files, w.align, ds.DS_PLAN_STRICT | ds.DS_PLAN_CHECK_MEMORY)
    eng = ds.ds_engine_create(4 * MiB, 1 * MiB, 2 * MiB, 2, 0, 0, 0)   # ring smaller than the image
    s = torch.cuda.current_stream().cuda_stream
    ck_paths = [str(tmp_path / f"rank0_{f}.ckpt") for f in range(n_files)]
    raw_paths = [str(tmp_path / f"rank0_{f}.img") for f in range(n_files)]
    try:
        # the image itself, straight from the kernel
        out = torch.full((total,), 0xFF, dtype=torch.uint8, device="cuda")
        ds.ds_pack(plan, out.data_ptr(), 0, total, s)
        torch.cuda.synchronize()
        assert gu.first_mismatch(out.cpu().numpy(), want_image) is None
        print("[step] image of the plan == the files' images one behind the other", flush=True)

        # one snapshot into seven checkpoint files, objects appended meanwhile
        ev = ds.ds_snapshot_async(eng, plan, s)
        parts = [ds.ds_ckpt_create_part(ck_paths[f], plan, f, file_flags) for f in range(n_files)]
        ds.ds_ckpt_flush_snapshot_parts(parts, ev, 3)
        appends = [[(1, b"file %d" % f), (2, bytes(range(f + 1)))] for f in range(n_files)]
        for f, ck in enumerate(parts):
            for oid, data in appends[f]:
                ds.ds_ckpt_append(ck, oid, data)
        with pytest.raises(ds.DsError) as e:                           # once per snapshot
            ds.ds_ckpt_flush_snapshot_parts(parts, ev, 3)
        assert e.value.code == ds.DS_ESTATE
        ds.ds_event_wait_on_stream(ev, s)
        arena.fill_(0xA5)                                              # the update phase may overwrite everything
        torch.cuda.synchronize()
        for ck in reversed(parts):                                     # any order
            ds.ds_ckpt_finish(ck)
        ds.ds_event_wait(ev)
        st = ds.ds_event_stats(ev)
        ds.ds_event_destroy(ev)
        assert st["n_pack_launches"] == -(-total // (2 * MiB))
        tensors = [(sh.tensor_id, W.DTYPES[sh.dtype][0], tuple(sh.shape), o, sh.nbytes)
                   for sh, o in zip(w.shards, offs)]
        want_files = fmt.build_rank_files(w.align, want_image.tobytes(), tensors, file_of, n_files, appends)
        for f in range(n_files):
            assert open(ck_paths[f], "rb").read() == want_files[f], f
        print("[step] every checkpoint file == the oracle's file of its shards", flush=True)

        # ONE restore of the rank out of all files
        readers = [ds.ds_ckpt_open(p) for p in ck_paths]
        rev = ds.ds_ckpt_restore_parts(readers, eng, plan, 3, file_flags & ds.DS_FILE_DIRECT, s)
        ds.ds_event_wait(rev)
        ds.ds_event_destroy(rev)
        with pytest.raises(ds.DsError) as e:                           # files in the wrong order are refused
            ds.ds_ckpt_restore_parts(readers[1:] + readers[:1], eng, plan, 3, 0, s)
        assert e.value.code == ds.DS_EFORMAT
        for r in readers:
            ds.ds_ckpt_close(r)
        mirror = w.arena.copy()
        try:
            w.arena[:] = 0xA5
            for f, (t, k) in enumerate(tabs):
                orc.unpack(t, k, alone[f])
            assert gu.first_mismatch(arena.cpu().numpy(), w.arena) is None
        finally:
            w.arena[:] = mirror
        print("[step] restore out of all files == the oracle's", flush=True)

        # the plain flush into several files, and the restore out of them
        ev = ds.ds_snapshot_async(eng, plan, s)
        fl = ds.ds_flush_start_files(ev, raw_paths, 2, file_flags)
        ds.ds_event_wait_on_stream(ev, s)
        arena.fill_(0x5A)
        nbytes, _ = ds.ds_flush_wait(fl)
        ds.ds_event_wait(ev)
        ds.ds_event_destroy(ev)
        assert nbytes == total
        for f in range(n_files):
            assert open(raw_paths[f], "rb").read() == alone[f].tobytes(), f
        with pytest.raises(ds.DsError) as e:                           # one path per file of the plan
            ds.ds_restore_from_files(eng, plan, raw_paths[:-1], 2, 0, s)
        assert e.value.code == ds.DS_EINVAL
        rev = ds.ds_restore_from_files(eng, plan, raw_paths, 2, file_flags & ds.DS_FILE_DIRECT, s)
        ds.ds_event_wait(rev)
        ds.ds_event_destroy(rev)
        try:
            w.arena[:] = 0x5A
            for f, (t, k) in enumerate(tabs):
                orc.unpack(t, k, alone[f])
            assert gu.first_mismatch(arena.cpu().numpy(), w.arena) is None
        finally:
            w.arena[:] = mirror
        # a whole-image flush of the same plan into ONE file is still the image
        ev = ds.ds_snapshot_async(eng, plan, s)
        one = str(tmp_path / "rank0_all.img")
        fl = ds.ds_flush_start(ev, one, 2, file_flags)
        ds.ds_event_wait_on_stream(ev, s)
        ds.ds_flush_wait(fl)
        ds.ds_event_wait(ev)
        ds.ds_event_destroy(ev)
        assert open(one, "rb").read() == want_image.tobytes()
    finally:
        ds.ds_engine_destroy(eng)
        torch.cuda.synchronize()
        ds.ds_plan_destroy(plan)


def test_flush_io_error_does_not_stall_the_snapshot():
    """Writers that fail (/dev/full: ENOSPC) still hand every ring slot back, so the
    snapshot runs to its end; the flush reports DS_EIO with the errno."""
    import os
    if not os.path.exists("/dev/full"):
        pytest.skip("no /dev/full here")
    ds, orc, gu, torch = _mods()
    w = W.fragmentation(1200, max_bytes=1 << 16, seed=95)
    print("[case] flush error path", flush=True)
    dw = gu.DeviceWorkload(w)
    eng = ds.ds_engine_create(4 * MiB, 1 * MiB, 4 * MiB, 2, 0, 0, 2)      # ring smaller than the image
    s = torch.cuda.current_stream().cuda_stream
    try:
        for fflags in (0, ds.DS_FILE_URING):
            ev = ds.ds_snapshot_async(eng, dw.plan, s)
            fl = ds.ds_flush_start(ev, "/dev/full", 2, fflags)
            ds.ds_event_wait_on_stream(ev, s)
            with pytest.raises(ds.DsError) as e:
                ds.ds_flush_wait(fl)
            assert e.value.code == ds.DS_EIO and ds.ds_last_errno() == 28
            ds.ds_event_wait(ev)                  # the snapshot itself completed
            ds.ds_event_destroy(ev)
        # and the engine is usable afterwards
        ev = ds.ds_snapshot_async(eng, dw.plan, s)
        n = 0
        while True:
            ch = ds.ds_snapshot_next_chunk(ev)
            if ch is None:
                break
            n += ch[2]
            ds.ds_snapshot_release_chunk(ev, ch[0])
        assert n == dw.total
        ds.ds_event_wait(ev)
        ds.ds_event_destroy(ev)
    finally:
        ds.ds_engine_destroy(eng)
        dw.close()


def test_flush_to_several_files_with_one_that_fails(tmp_path):
    """One of the files of a plan of several cannot be written (/dev/full: ENOSPC): the flush reports DS_EIO
    with the errno, every ring slot still goes back (pieces of a slot that lie in other files included), so
    the snapshot runs to its end, and the next flush of the same plan into good files is byte-exact."""
    import os
    if not os.path.exists("/dev/full"):
        pytest.skip("no /dev/full here")
    ds, orc, gu, torch = _mods()
    w = W.fragmentation(1200, max_bytes=1 << 16, seed=96)
    n = len(w.shards)
    print("[case] several files, one fails", flush=True)
    arena = torch.from_numpy(w.arena).to("cuda")
    file_of = [min(3, (4 * i) // n) for i in range(n)]
    descs = ds.make_descs(w.shards, arena.data_ptr())
    regions, total = ds.ds_layout_assign_files(descs, file_of, n, 4, w.align)
    plan = ds.ds_plan_create_files(descs, file_of, n, 4, w.align, ds.DS_PLAN_STRICT | ds.DS_PLAN_CHECK_MEMORY)
    eng = ds.ds_engine_create(4 * MiB, 1 * MiB, 4 * MiB, 2, 0, 0, 1)       # ring smaller than the image
    s = torch.cuda.current_stream().cuda_stream
    good = [str(tmp_path / f"f{k}.img") for k in range(4)]
    try:
        for fflags in (0, ds.DS_FILE_DIRECT, ds.DS_FILE_URING):
            ev = ds.ds_snapshot_async(eng, plan, s)
            fl = ds.ds_flush_start_files(ev, [good[0], "/dev/full", good[2], good[3]], 3, fflags)
            ds.ds_event_wait_on_stream(ev, s)
            with pytest.raises(ds.DsError) as e:
                ds.ds_flush_wait(fl)
            assert e.value.code == ds.DS_EIO and ds.ds_last_errno() == 28
            ds.ds_event_wait(ev)                  # the snapshot itself completed
            ds.ds_event_destroy(ev)
        with pytest.raises(ds.DsError) as e:      # a file that cannot be created: nothing is started
            ds.ds_flush_start_files(ev := ds.ds_snapshot_async(eng, plan, s), [good[0], str(tmp_path / "no" / "dir"),
                                                                             good[2], good[3]], 2, 0)
        assert e.value.code == ds.DS_EIO and ds.ds_last_errno() == 2
        fl = ds.ds_flush_start_files(ev, good, 2, ds.DS_FILE_DIRECT)       # the same snapshot, now into good files
        ds.ds_event_wait_on_stream(ev, s)
        assert ds.ds_flush_wait(fl)[0] == total
        ds.ds_event_wait(ev)
        ds.ds_event_destroy(ev)
        for f in range(4):
            sub = [sh for sh, g in zip(w.shards, file_of) if g == f]
            t = orc.table(sub, w.arena.ctypes.data)
            assert orc.layout(t, len(sub), w.align) == regions[f]
            assert open(good[f], "rb").read() == orc.pack(t, len(sub), regions[f], threads=4).tobytes(), f
    finally:
        ds.ds_engine_destroy(eng)
        torch.cuda.synchronize()
        ds.ds_plan_destroy(plan)


def test_timeline_trace_of_a_snapshot():
    """An engine with DS_ENGINE_TRACE times every chunk copy: the records cover the
    image exactly once per tier, every copy starts after the gather that filled its
    staging slot has ended, and copies on one stream do not overlap."""
    ds, orc, gu, torch = _mods()
    w = W.fragmentation(1500, max_bytes=1 << 17, seed=97)
    print("[case] timeline trace", flush=True)
    dw = gu.DeviceWorkload(w)
    eng = ds.ds_engine_create(64 * MiB, 2 * MiB, 16 * MiB, 2, 0, ds.DS_ENGINE_AUTO_RELEASE | ds.DS_ENGINE_TRACE, 1)
    s = torch.cuda.current_stream().cuda_stream
    try:
        ev = ds.ds_snapshot_async(eng, dw.plan, s)
        try:
            ds.ds_event_trace(ev)              # most likely still in flight
        except ds.DsError as e:
            assert e.code == ds.DS_EBUSY
        ds.ds_event_wait(ev)
        recs = ds.ds_event_trace(ev)
        st = ds.ds_event_stats(ev)
        gathers = [r for r in recs if r["kind"] == 0]
        copies = [r for r in recs if r["kind"] == 1]
        assert len(gathers) == st["n_pack_launches"] == -(-dw.total // (16 * MiB))
        assert len(copies) == st["n_copies"]
        for tier in (gathers, copies):
            at = 0
            for r in tier:
                assert r["file_off"] == at and r["len"] > 0 and r["end_ms"] >= r["begin_ms"] >= 0
                at += r["len"]
            assert at == dw.total
        for c in copies:
            g = gathers[c["file_off"] // (16 * MiB)]
            assert c["begin_ms"] >= g["end_ms"] - 1e-3
        for a, b in zip(copies, copies[1:]):
            assert b["begin_ms"] >= a["end_ms"] - 1e-3            # one copy stream: in order
        assert abs(max(c["end_ms"] for c in copies) - st["total_ms"]) < 5.0
        ds.ds_event_destroy(ev)
        # without the flag only the gathers are reported
        eng2 = ds.ds_engine_create(64 * MiB, 2 * MiB, 16 * MiB, 2, 0, ds.DS_ENGINE_AUTO_RELEASE, 1)
        ev = ds.ds_snapshot_async(eng2, dw.plan, s)
        ds.ds_event_wait(ev)
        assert {r["kind"] for r in ds.ds_event_trace(ev)} == {0}
        ds.ds_event_destroy(ev)
        ds.ds_engine_destroy(eng2)
    finally:
        ds.ds_engine_destroy(eng)
        dw.close()


def test_two_engines_from_two_threads():
    """Two engines, each driven by its own thread with its own plan and stream,
    at the same time: nothing is shared but the device, so both images must be
    the oracle's."""
    import threading
    ds, orc, gu, torch = _mods()
    ws = [W.fragmentation(1200, max_bytes=1 << 17, seed=201), W.llama_rank("mini", 256, 704, 4, 2, 1024, 2, 4, 8, seed=7, workers=2)]
    print("[case] two engines", flush=True)
    wants = [gu.oracle_image(w)[0] for w in ws]
    dws = [gu.DeviceWorkload(w) for w in ws]
    torch.cuda.synchronize()
    results, errors = [None, None], []

    def run(i):
        try:
            torch.cuda.set_device(0)
            st = torch.cuda.Stream()
            eng = ds.ds_engine_create(8 * MiB, 1 * MiB, 8 * MiB, 2, 0, 0, 2)
            try:
                for rep in range(3):
                    ev = ds.ds_snapshot_async(eng, dws[i].plan, st.cuda_stream)
                    got = np.empty(dws[i].total, dtype=np.uint8)
                    while True:
                        ch = ds.ds_snapshot_next_chunk(ev)
                        if ch is None:
                            break
                        ptr, off, ln = ch
                        ctypes.memmove(got.ctypes.data + off, ptr, ln)
                        ds.ds_snapshot_release_chunk(ev, ptr)
                    ds.ds_event_wait(ev)
                    ds.ds_event_destroy(ev)
                    assert gu.first_mismatch(got, wants[i]) is None, (i, rep)
                results[i] = True
            finally:
                ds.ds_engine_destroy(eng)
        except BaseException as e:   # noqa: BLE001 - reported in the main thread
            errors.append((i, repr(e)))

    import ctypes
    ts = [threading.Thread(target=run, args=(i,)) for i in range(2)]
    for t in ts:
        t.start()
    for t in ts:
        t.join()
    for dw in dws:
        dw.close()
    assert not errors, errors
    assert results == [True, True]
