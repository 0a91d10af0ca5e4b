#!/usr/bin/env python3
"""Benchmark of the snapshot hot path on one MI355X.

A step = one lazy snapshot of one rank's state: request on the compute stream,
gather into device staging, chunked copies into the pinned host ring, and the
gate before the (here empty) update phase; the step ends when the whole image
is resident in the host ring.  Steps run one after the other, so the gather
kernel of a step runs alone on the GPU (as it does in training, where an
iteration is longer than a snapshot).  `pipelined_GBps` reports the same loop
without the per-step wait (the gather of step i+1 under the copies of step i).
The inputs are resident in HBM before the timed region.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llama7b]

Prints ONE JSON line.  The top-level fields are the headline workload's (the
Llama-7B rank: the state the overlap configuration is quoted on): `value` is
payload GB/s of the whole step (link-bound); `roofline` is the gather kernel
against the HBM peak, timed with HIP events on the stream it runs on;
`cpu_baseline` is the CPU oracle's pack of the same workload on this machine's host
cores.  `per_workload` repeats value / roofline / link fraction / capture time /
parity for all four shard sets, each measured and byte-compared with the oracle
in this same run; `cap_binding` holds the runs in which the host ring and the
device staging are smaller than the image; `overlap` the snapshots under the
GEMM stream at several compute windows; `experiments` the capture variants that
are measured, not shipped.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
MiB = 1 << 20
GiB = 1 << 30
METRIC = "snapshot GB/s/GPU (pack+D2H to pinned host)"

WORKLOADS = {
    "tiny_gpt": "configs[0] tiny GPT-style state, 118 shards",
    "llama7b": "configs[1] Llama-7B rank (TP=4, PP=4, ZeRO-1 DP=8), 76 shards",
    "fragmentation": "configs[2] fragmentation stress, 20000 shards",
    "llama70b": "configs[3] Llama-2-70B rank (TP=8, PP=4, ZeRO-1 DP=8), 184 shards",
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Ctx:
    """What every leg needs: the modules, the device, the stream, the options."""

    def __init__(self, args):
        import numpy as np
        import torch

        import paper_2601_16956_amd as ds
        import workloads as W
        assert torch.cuda.is_available(), "needs the MI355X"
        self.np, self.torch, self.ds, self.W, self.args = np, torch, ds, W, args
        self.dev = torch.device("cuda:0")
        torch.cuda.set_device(self.dev)
        self.stream = torch.cuda.current_stream().cuda_stream
        cores = len(os.sched_getaffinity(0))
        self.cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))
        self.link_d2h = self.link_h2d = 0.0

    def timed(self, fn, reps=20, warm=3):
        """(median, best) milliseconds of fn, each call bracketed by events on the current stream."""
        torch = self.torch
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        pairs = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            pairs.append((a, b))
        torch.cuda.synchronize()
        ts = sorted(a.elapsed_time(b) for a, b in pairs)
        return ts[len(ts) // 2], ts[0]

    def engine(self, cfg, flags=None, grid_limit=0):
        ds = self.ds
        return ds.ds_engine_create(cfg["ring"], cfg["chunk"], cfg["slot"], cfg["slots"], grid_limit,
                                   ds.DS_ENGINE_AUTO_RELEASE if flags is None else flags, cfg["copy_streams"], cfg["first"])


def engine_cfg(args, **over):
    cfg = {"ring": args.ring_bytes, "chunk": args.chunk_bytes, "slot": args.stage_slot_bytes, "slots": args.stage_slots,
           "copy_streams": args.copy_streams, "first": args.first_launch_bytes}
    cfg.update(over)
    return cfg


def engine_json(cfg):
    return {"host_ring_bytes": cfg["ring"], "d2h_chunk_bytes": cfg["chunk"], "stage_slot_bytes": cfg["slot"],
            "stage_slots": cfg["slots"], "copy_streams": cfg["copy_streams"], "first_launch_bytes": cfg["first"]}


def measure_link(c: Ctx):
    """Measured link peak: best of 10 x 1 GiB contiguous device -> pinned host, and 6 the other way."""
    torch = c.torch
    probe_dev = torch.empty(GiB, dtype=torch.uint8, device=c.dev).random_(0, 255)
    probe_host = torch.empty(GiB, dtype=torch.uint8, pin_memory=True)
    for i in range(12):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        probe_host.copy_(probe_dev, non_blocking=True)
        b.record()
        torch.cuda.synchronize()
        if i >= 2:
            c.link_d2h = max(c.link_d2h, GiB / (a.elapsed_time(b) * 1e-3) / 1e9)
    for i in range(8):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        probe_dev.copy_(probe_host, non_blocking=True)
        b.record()
        torch.cuda.synchronize()
        if i >= 2:
            c.link_h2d = max(c.link_h2d, GiB / (a.elapsed_time(b) * 1e-3) / 1e9)
    log(f"[bench] measured link peak: D2H {c.link_d2h:.1f} GB/s, H2D {c.link_h2d:.1f} GB/s")


class Loaded:
    """A workload generated, uploaded and planned."""

    def __init__(self, c: Ctx, name: str):
        ds, torch = c.ds, c.torch
        t0 = time.time()
        self.name = name
        self.w = c.W.by_name(name, workers=c.cores)
        w = self.w
        log(f"[bench] generated {w.name}: {len(w.shards)} shards, payload {w.payload_bytes / 1e9:.3f} GB, "
            f"arena {w.arena.size / 1e9:.3f} GB in {time.time() - t0:.1f}s")
        self.arena = torch.from_numpy(w.arena).to(c.dev)
        self.n = len(w.shards)
        self.descs = ds.make_descs(w.shards, self.arena.data_ptr())
        self.total = ds.ds_layout_assign(self.descs, self.n, w.align)
        t0 = time.perf_counter()
        self.plan = ds.ds_plan_create(self.descs, self.n, w.align, ds.DS_PLAN_STRICT | ds.DS_PLAN_CHECK_MEMORY)
        self.plan_ms = (time.perf_counter() - t0) * 1e3
        self.info = ds.ds_plan_info(self.plan)
        self.payload = self.info["payload_bytes"]
        self.algo_bytes = self.payload + self.total   # one gather launch: payload read once, image written once
        self.want = None                              # the oracle's image, once the parity leg has made it

    def close(self, c: Ctx):
        c.torch.cuda.synchronize()
        c.ds.ds_plan_destroy(self.plan)
        self.plan = None
        self.arena = None
        self.want = None
        self.w = None


def settle(c: Ctx):
    """Gives a workload's device memory back and waits a moment.  Measured: for some hundreds of milliseconds
    after gigabytes of device memory have been freed, device-to-host copies queued back to back run at half
    their rate (a 27 MB copy takes 1.04 instead of 0.49 ms; one second later all is as in a fresh process),
    which would be charged to the next workload's pipelined figure."""
    c.torch.cuda.empty_cache()
    time.sleep(1.0)


def write_manifest(c: Ctx, L: Loaded):
    """What this run's input was, so that it can be rebuilt: generator, seed, and the shard table as realised."""
    args, w = c.args, L.w
    path = args.manifest or os.path.join(ROOT, "bench_out", f"manifest_{L.name}.json")
    if path == "-":
        return None
    try:
        os.makedirs(os.path.dirname(os.path.abspath(path)), exist_ok=True)
        with open(path, "w") as f:
            json.dump({"workload": L.name, "generator": f"workloads.by_name({L.name!r})",
                       "name": w.name, "seed": w.seed, "align": w.align, "shards": L.n, "payload_bytes": L.payload,
                       "image_bytes": L.total, "arena_bytes": int(w.arena.size), "notes": w.notes,
                       "table": [{"name": sh.name, "dtype": sh.dtype, "shape": list(sh.shape),
                                  "strides": list(sh.strides), "byte_offset": sh.byte_offset,
                                  "tensor_id": sh.tensor_id, "file_offset": int(L.descs[i].file_offset),
                                  "nbytes": sh.nbytes} for i, sh in enumerate(w.shards)]}, f)
        return os.path.relpath(path, ROOT)
    except OSError as e:
        log(f"[bench] manifest not written: {e}")
        return None


def snapshot_steps(c: Ctx, eng, plan, k, pipelined=False):
    ds = c.ds
    evs = []
    for _ in range(k):
        ev = ds.ds_snapshot_async(eng, plan, c.stream)
        ds.ds_event_wait_on_stream(ev, c.stream)       # gate before the (empty) update phase
        if not pipelined:
            ds.ds_event_wait(ev)                       # the whole image is in the host ring
        evs.append(ev)
    for ev in evs:
        ds.ds_event_wait(ev)
    return evs


def traffic_from_profile(c: Ctx, name: str):
    """HBM bytes per gather launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, from the committed
    summary of that run -- only if the summary was taken with the kernel sources that are in use now."""
    path = os.path.join(ROOT, "profiles", f"pmc_traffic_{name}.md")
    if not os.path.exists(path):
        return None, {"note": "no counter profile committed for this workload"}
    text = open(path).read()
    m = re.search(r"traffic_bytes_per_launch\s*=\s*(\d+)", text)
    d = re.search(r"kernel_source_digest\s*=\s*([0-9a-f]+)", text)
    now = c.ds.kernel_source_digest()
    src = {"file": os.path.relpath(path, ROOT), "profile_kernel_source_digest": d.group(1) if d else None,
           "kernel_source_digest": now,
           "scaling": "counters scaled to ds_copy_probe of known size: relative to that probe, not absolute"}
    if not m or not d or d.group(1) != now:
        src["note"] = "the profile was taken with other kernel sources: traffic not reported"
        return None, src
    return int(m.group(1)), src


def timed_region(c: Ctx, L: Loaded, cfg, steps, warmup, extras=True):
    """K snapshots back to back, each gated and waited for; returns the bench fields of that region.  With
    `extras` also one isolated snapshot and the same steps without the per-step wait."""
    ds, torch = c.ds, c.torch
    eng = c.engine(cfg)
    try:
        for ev in snapshot_steps(c, eng, L.plan, warmup):
            ds.ds_event_destroy(ev)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        evs = snapshot_steps(c, eng, L.plan, steps)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        pack_ms = copy_ms = capture_ms = submit_ms = 0.0
        launches = 0
        for ev in evs:
            st = ds.ds_event_stats(ev)
            pack_ms += st["pack_ms"]
            copy_ms += st["copy_ms"]
            capture_ms += st["capture_ms"]
            submit_ms += st["submit_host_ms"]
            launches += st["n_pack_launches"]
            ds.ds_event_destroy(ev)
        latency_ms, one, pipelined = 0.0, {"total_ms": 0.0}, 0.0
        if extras:
            # one isolated snapshot: request -> whole image resident in the host ring
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ev = ds.ds_snapshot_async(eng, L.plan, c.stream)
            ds.ds_event_wait(ev)
            latency_ms = (time.perf_counter() - t0) * 1e3
            one = ds.ds_event_stats(ev)
            ds.ds_event_destroy(ev)
            # the same steps without the per-step wait (once untimed: the first time that many snapshots are in
            # flight at once, the runtime and the engine create the events and queue entries they then reuse)
            for ev in snapshot_steps(c, eng, L.plan, steps if L.total < (256 << 20) else min(3, steps), pipelined=True):
                ds.ds_event_destroy(ev)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            pevs = snapshot_steps(c, eng, L.plan, steps, pipelined=True)
            torch.cuda.synchronize()
            pipelined = L.payload * steps / (time.perf_counter() - t0) / 1e9
            for ev in pevs:
                ds.ds_event_destroy(ev)
    finally:
        ds.ds_engine_destroy(eng)
    achieved = L.algo_bytes * steps / (pack_ms * 1e-3) / 1e9 if pack_ms > 0 else 0.0
    traffic, traffic_src = traffic_from_profile(c, L.name)
    d2h = L.total * steps / (copy_ms * 1e-3) / 1e9 if copy_ms > 0 else 0.0
    return {
        "value": round(L.payload * steps / elapsed / 1e9, 3), "steps": steps, "warmup": warmup,
        "ms_per_step": round(elapsed * 1e3 / steps, 3),
        "roofline": {
            "bound": "hbm", "kernel": "ds_move_kernel<pack>", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
            "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic, "traffic_source": traffic_src,
            "launches": launches, "avg_launch_ms": round(pack_ms / max(launches, 1), 4),
            "algorithmic_bytes_per_launch": L.algo_bytes * steps // max(launches, 1)},
        "d2h": {"achieved_GBps": round(d2h, 2), "link_peak_measured_GBps": round(c.link_d2h, 2),
                "frac": round(d2h / c.link_d2h, 4) if c.link_d2h else None,
                "end_to_end_frac_of_link": round(L.payload * steps / elapsed / 1e9 / c.link_d2h, 4) if c.link_d2h else None},
        "snapshot_latency_ms": round(latency_ms, 3), "one_total_ms": one["total_ms"],
        "pipelined_GBps": round(pipelined, 3),
        "capture_ms": round(capture_ms / steps, 3),          # request -> tensors may be mutated
        "submit_host_ms": round(submit_ms / steps, 4),       # host time inside ds_snapshot_async
    }


def standalone(c: Ctx, L: Loaded):
    """Gather and scatter alone, whole image, device to device; the plain copy probe and the runtime's copy."""
    ds, torch = c.ds, c.torch
    total = L.total
    image_dev = torch.empty(max(total, 16), dtype=torch.uint8, device=c.dev)
    pack_med, pack_best = c.timed(lambda: ds.ds_pack(L.plan, image_dev.data_ptr(), 0, total, c.stream))
    unpack_med, _ = c.timed(lambda: ds.ds_unpack(L.plan, image_dev.data_ptr(), 0, total, c.stream))
    copy_src = torch.empty_like(image_dev)
    nprobe = total & ~15
    probe_med, _ = c.timed(lambda: ds.ds_copy_probe(image_dev.data_ptr(), copy_src.data_ptr(), nprobe, c.stream))
    dtod_med, _ = c.timed(lambda: copy_src.copy_(image_dev))      # the runtime's own device-to-device copy
    del copy_src, image_dev
    return {
        "pack_ms": round(pack_med, 4), "pack_GBps": round(L.algo_bytes / pack_med / 1e6, 1),
        "pack_best_GBps": round(L.algo_bytes / pack_best / 1e6, 1),
        "unpack_ms": round(unpack_med, 4), "unpack_GBps": round(2 * L.payload / unpack_med / 1e6, 1),
        "copy_probe_GBps": round(2 * nprobe / probe_med / 1e6, 1),    # plain copy, same shape: the ceiling
        "runtime_d2d_copy_GBps": round(2 * total / dtod_med / 1e6, 1),   # torch copy_ (hipMemcpy device to device)
        "pack_vs_copy_probe": round((L.algo_bytes / pack_med) / (2 * nprobe / probe_med), 4),
    }


def same_bytes(c: Ctx, a, b):
    np = c.np
    return a.size == b.size and all(np.array_equal(a[lo:lo + (1 << 28)], b[lo:lo + (1 << 28)]) for lo in range(0, a.size, 1 << 28))


def parity_and_cpu(c: Ctx, L: Loaded, cfg, want_baseline: bool):
    """This very run against the CPU oracle: the gathered image, the scatter of the oracle's image into a wiped
    arena (whole arena compared), and the same restore through the engine's pipeline.  With want_baseline the
    oracle's pack is also timed on this machine's host cores."""
    ds, torch, np = c.ds, c.torch, c.np
    from oracle import ds_oracle as orc
    w, n, total = L.w, L.n, L.total
    tab = orc.table(w.shards, w.arena.ctypes.data)
    assert orc.layout(tab, n, w.align) == total
    want = np.empty(total, dtype=np.uint8)
    orc.pack(tab, n, total, threads=c.cores, out=want)          # also faults the pages in
    cpu_baseline = None
    if want_baseline:
        runs = []
        for _ in range(3):
            t0 = time.perf_counter()
            orc.pack(tab, n, total, threads=c.cores, out=want)
            runs.append(time.perf_counter() - t0)
        t0 = time.perf_counter()
        orc.pack(tab, n, total, threads=1, out=want)
        single = time.perf_counter() - t0
        cpu_baseline = {
            "value": round(L.payload / sorted(runs)[1] / 1e9, 2), "unit": "GB/s", "cores": c.cores, "kind": "oracle",
            "sample": f"dso_pack_mt of the whole {L.name} image ({L.payload / 1e9:.2f} GB), median of 3 runs "
                      f"after 1 warm-up, {c.cores} threads; single thread: {L.payload / single / 1e9:.2f} GB/s",
        }
    image_dev = torch.empty(max(total, 16), dtype=torch.uint8, device=c.dev)
    ds.ds_pack(L.plan, image_dev.data_ptr(), 0, total, c.stream)
    torch.cuda.synchronize()
    got = image_dev[:total].cpu().numpy()
    parity = "byte-exact vs CPU oracle" if same_bytes(c, got, want) else "MISMATCH vs CPU oracle"
    del got
    # restore: scatter the oracle's image back into a wiped arena, compare the whole arena
    keep = L.arena.clone()
    host_keep = w.arena.copy()
    L.arena.fill_(0xA5)
    image_dev[:total].copy_(torch.from_numpy(want))
    ds.ds_unpack(L.plan, image_dev.data_ptr(), 0, total, c.stream)
    torch.cuda.synchronize()
    back = L.arena.cpu().numpy()
    w.arena[:] = 0xA5
    orc.unpack(tab, n, want)
    parity += "; restore byte-exact" if same_bytes(c, back, w.arena) else "; restore MISMATCH"
    # the same restore through the pipeline: host image -> ring slots -> staging -> scatter
    eng = c.engine(cfg)
    try:
        L.arena.fill_(0xA5)
        rev = ds.ds_restore_begin(eng, L.plan, c.stream)
        while True:
            slot = ds.ds_restore_next_slot(rev)
            if slot is None:
                break
            ptr, off, ln = slot
            ctypes.memmove(ptr, want[off:off + ln].ctypes.data, ln)
            ds.ds_restore_submit(rev, ptr)
        ds.ds_event_wait(rev)
        ds.ds_event_destroy(rev)
        back = L.arena.cpu().numpy()
        parity += "; pipelined restore byte-exact" if same_bytes(c, back, w.arena) else "; pipelined restore MISMATCH"
    finally:
        ds.ds_engine_destroy(eng)
    L.arena.copy_(keep)
    w.arena[:] = host_keep
    del keep, back, host_keep, image_dev
    L.want = want
    return parity, cpu_baseline


def workload_entry(c: Ctx, L: Loaded, cfg, steps, warmup, want_baseline=False):
    """Everything `per_workload` reports for one shard set."""
    tr = timed_region(c, L, cfg, steps, warmup)
    sa = standalone(c, L)
    parity, cpu_baseline = ("not checked", None)
    if not c.args.no_cpu_baseline:
        parity, cpu_baseline = parity_and_cpu(c, L, cfg, want_baseline)
    entry = {"workload": f"{L.name}: {WORKLOADS[L.name]}", "shards": L.n, "payload_bytes": L.payload,
             "image_bytes": L.total, "align": L.w.align, "general_chunks": L.info["n_general_chunks"],
             "chunks": L.info["n_chunks"], "engine": engine_json(cfg),
             **{k: tr[k] for k in ("value", "steps", "warmup", "ms_per_step", "roofline", "d2h", "snapshot_latency_ms",
                                   "pipelined_GBps", "capture_ms", "submit_host_ms")},
             "plan_create_ms": round(L.plan_ms, 3), "standalone": sa, "parity": parity}
    log(f"[bench] {L.name}: {entry['value']} GB/s, gather {entry['roofline']['achieved']} GB/s "
        f"({entry['roofline']['frac']:.3f} of HBM peak), capture {entry['capture_ms']} ms, {parity}")
    return entry, tr, cpu_baseline


def cap_binding_run(c: Ctx, L: Loaded, cfg, steps, what):
    """A run in which the ring and/or the staging are smaller than the image, with a consumer thread that copies
    every chunk out (so the ring really fills and drains) and compares the image with the oracle's."""
    import threading
    ds, np = c.ds, c.np
    tr = timed_region(c, L, cfg, steps, min(2, c.args.warmup))
    exact = None
    if L.want is not None:
        eng = c.engine(cfg, flags=0)
        try:
            got = np.empty(L.total, dtype=np.uint8)
            ev = ds.ds_snapshot_async(eng, L.plan, c.stream)

            def consumer():
                while True:
                    ch = ds.ds_snapshot_next_chunk(ev)
                    if ch is None:
                        return
                    ptr, off, ln = ch
                    ctypes.memmove(got.ctypes.data + off, ptr, ln)
                    ds.ds_snapshot_release_chunk(ev, ptr)
            th = threading.Thread(target=consumer)
            th.start()
            ds.ds_event_wait_on_stream(ev, c.stream)
            th.join()
            ds.ds_event_wait(ev)
            ds.ds_event_destroy(ev)
            exact = same_bytes(c, got, L.want)
            del got
        finally:
            ds.ds_engine_destroy(eng)
    res = {"what": what, "workload": L.name, "image_bytes": L.total, "engine": engine_json(cfg),
           "value": tr["value"], "ms_per_step": tr["ms_per_step"], "steps": steps,
           "gather_GBps": tr["roofline"]["achieved"], "gather_frac_of_hbm_peak": tr["roofline"]["frac"],
           "gather_launches_per_snapshot": tr["roofline"]["launches"] // steps,
           "d2h_frac_of_link": tr["d2h"]["frac"], "capture_ms": tr["capture_ms"],
           "image_through_consumer_byte_exact_vs_oracle": exact}
    log(f"[bench] cap-binding run, {L.name}, {what}: {res['value']} GB/s, capture {res['capture_ms']} ms, "
        f"byte-exact {exact}")
    return res


def overlap_leg(c: Ctx, L: Loaded, cfg, one_total_ms):
    """configs[4]: snapshots every iteration under a bf16 8192^3 GEMM stream, with a mutating update behind the
    gate, at compute windows of 1.5, 1.0 and 0.5 snapshot times, and a stress point of a sixth of the first."""
    ds, torch, args = c.ds, c.torch, c.args
    M = 8192
    A = torch.randn(M, M, device=c.dev, dtype=torch.bfloat16)
    B = torch.randn(M, M, device=c.dev, dtype=torch.bfloat16)
    C = torch.empty(M, M, device=c.dev, dtype=torch.bfloat16)
    for _ in range(5):
        torch.matmul(A, B, out=C)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(20):
        torch.matmul(A, B, out=C)
    b.record()
    torch.cuda.synchronize()
    gemm_ms = a.elapsed_time(b) / 20
    eng = c.engine(cfg)
    state = {}

    def loop(with_snapshots: bool, G: int, eng=eng, iters=None):
        iters = iters or args.gemm_iters
        evs, prev = [], None
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        state["gate_host_ms"] = 0.0
        torch.cuda.synchronize()
        w0 = time.perf_counter()
        a.record()
        for _ in range(iters):
            for _ in range(G):                                # state is only read here
                torch.matmul(A, B, out=C)
            if prev is not None:
                g0 = time.perf_counter()
                ds.ds_event_wait_on_stream(prev, c.stream)    # the lazy gate
                state["gate_host_ms"] += (time.perf_counter() - g0) * 1e3
            L.arena.add_(1)                                   # the mutating update phase
            if with_snapshots:
                prev = ds.ds_snapshot_async(eng, L.plan, c.stream)
                evs.append(prev)
        b.record()
        torch.cuda.synchronize()
        for ev in evs:
            ds.ds_event_wait(ev)
            ds.ds_event_destroy(ev)
        state["wall_ms"] = (time.perf_counter() - w0) * 1e3   # until the last snapshot is in the host ring
        return a.elapsed_time(b)

    def window(factor):
        G = max(1, int(round(factor * one_total_ms / gemm_ms)))
        loop(True, G)
        base = min(loop(False, G) for _ in range(2))
        with_s = min(loop(True, G) for _ in range(2))
        blocked = max(with_s - base, 1e-6) / args.gemm_iters
        return {"window_in_snapshot_times": factor, "gemms_per_iter": G, "ms_without_snapshots": round(base, 2),
                "ms_with_snapshots": round(with_s, 2), "slowdown_pct": round(100.0 * (with_s - base) / base, 2),
                "blocked_ms_per_iter": round(blocked, 4),
                # the paper's measure (Sec. VI-D): checkpoint size over the time training is blocked by it
                "effective_checkpoint_GBps": round(L.payload / blocked / 1e6, 1),
                "gate_call_host_ms_per_iter": round(state["gate_host_ms"] / args.gemm_iters, 4),
                "snapshot_GBps_sustained": round(L.payload * args.gemm_iters / state["wall_ms"] / 1e6, 2)}

    try:
        wins = [window(f) for f in (1.5, 1.0, 0.5)]
        head = wins[0]
        out = {"gemm": "bf16 8192x8192x8192 (torch.matmul)", "gemm_ms": round(gemm_ms, 3),
               "gemm_tflops": round(2 * M ** 3 / gemm_ms / 1e9, 1), "iters": args.gemm_iters,
               "engine": engine_json(cfg),
               **{k: head[k] for k in ("gemms_per_iter", "ms_without_snapshots", "ms_with_snapshots", "slowdown_pct",
                                       "blocked_ms_per_iter", "effective_checkpoint_GBps", "gate_call_host_ms_per_iter")},
               "windows": wins}
        # stress point: a compute window far shorter than one snapshot, so every gate stalls and the
        # loop runs at the pace of the link (back-pressure of the ring and the staging slots)
        Gs = max(1, head["gemms_per_iter"] // 6)
        base_s = min(loop(False, Gs) for _ in range(2))
        with_ss = loop(True, Gs)
        out["stress"] = {
            "gemms_per_iter": Gs, "ms_without_snapshots": round(base_s, 2), "ms_with_snapshots": round(with_ss, 2),
            "wall_ms_until_last_snapshot_done": round(state["wall_ms"], 2),
            "snapshot_GBps_sustained": round(L.payload * args.gemm_iters / state["wall_ms"] / 1e6, 2),
            "note": "compute window 1/6 of the first: the gate and the staging slots make the loop wait for the link"}
    except BaseException:
        ds.ds_engine_destroy(eng)
        raise
    return out, loop, (A, B, C), head, eng


def experiments_leg(c: Ctx, L: Loaded, cfg, loop, gemm, head, full: bool):
    """Capture variants that are measured, not shipped; each with its byte-exactness against the oracle's image
    (where the oracle's image of this run is at hand)."""
    ds, torch, args = c.ds, c.torch, c.args
    total, payload = L.total, L.payload
    out = {}
    base = head["ms_without_snapshots"] if head else None
    G = head["gemms_per_iter"] if head else None
    pristine = torch.from_numpy(L.w.arena)

    def image_is_oracles(host_tensor):
        if L.want is None:
            return None
        return same_bytes(c, host_tensor[:total].numpy(), L.want)

    # (1) The gather limited to a few resident work-groups: does a slower, narrower gather disturb the GEMM
    # stream less?
    if loop is not None:
        rows = []
        for limit in ((4096, 1024, 256) if full else (1024, 256)):
            eng_x = c.engine(cfg, grid_limit=limit)
            try:
                ev = ds.ds_snapshot_async(eng_x, L.plan, c.stream)
                ds.ds_event_wait(ev)
                st = ds.ds_event_stats(ev)
                ds.ds_event_destroy(ev)
                loop(True, G, eng_x)
                with_x = min(loop(True, G, eng_x) for _ in range(2))
            finally:
                ds.ds_engine_destroy(eng_x)
            exact = None
            if L.want is not None:
                ds.ds_config_set("grid_limit", limit)
                img = torch.empty(max(total, 16), dtype=torch.uint8, device=c.dev)
                L.arena.copy_(pristine)                  # the loop has mutated the tensors
                ds.ds_pack(L.plan, img.data_ptr(), 0, total, c.stream)
                torch.cuda.synchronize()
                ds.ds_config_set("grid_limit", 0)
                exact = same_bytes(c, img[:total].cpu().numpy(), L.want)
                del img
            rows.append({"resident_workgroups": limit, "gather_ms": round(st["pack_ms"], 3),
                         "capture_ms": round(st["capture_ms"], 3),
                         "slowdown_pct": round(100.0 * (with_x - base) / base, 2), "byte_exact_vs_oracle": exact})
        out["grid_limited_gather"] = {"unlimited_slowdown_pct": head["slowdown_pct"], "rows": rows}

    # (2) No staging and no copy: the gather writes straight into pinned host memory over the link.
    host_img = torch.empty(max(total, 16), dtype=torch.uint8, pin_memory=True)
    d_med, d_best = c.timed(lambda: ds.ds_pack(L.plan, host_img.data_ptr(), 0, total, c.stream), reps=5, warm=1)
    L.arena.copy_(pristine)
    ds.ds_pack(L.plan, host_img.data_ptr(), 0, total, c.stream)
    torch.cuda.synchronize()
    direct = {
        "ms": round(d_med, 3), "GBps": round(payload / d_med / 1e6, 2), "best_GBps": round(payload / d_best / 1e6, 2),
        "byte_exact_vs_oracle": image_is_oracles(host_img),
        "note": "the kernel holds the tensors for the whole transfer, so the gate opens after this time, "
                "not after the 0.5 ms of the staged gather; resident_workgroups 0 = one work-group per chunk"}
    if loop is not None:
        A, B, C = gemm
        side = torch.cuda.Stream()                    # default priority
        iters = args.gemm_iters if full else max(4, args.gemm_iters // 3)

        def loop_direct():
            prev = None
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            a.record()
            for _ in range(iters):
                for _ in range(G):
                    torch.matmul(A, B, out=C)
                if prev is not None:
                    torch.cuda.current_stream().wait_event(prev)   # the gate: the whole transfer
                L.arena.add_(1)
                req = torch.cuda.Event()
                req.record()
                side.wait_event(req)
                ds.ds_pack(L.plan, host_img.data_ptr(), 0, total, side.cuda_stream)
                prev = torch.cuda.Event()
                prev.record(side)
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b)

        base_d = base * iters / args.gemm_iters
        direct["under_gemms"] = []
        for limit in ((0, 1024, 256, 64, 16) if full else (0, 64)):
            ds.ds_config_set("grid_limit", limit)
            x_med, _ = c.timed(lambda: ds.ds_pack(L.plan, host_img.data_ptr(), 0, total, c.stream), reps=3, warm=1)
            loop_direct()
            with_d = min(loop_direct() for _ in range(2))
            direct["under_gemms"].append({
                "resident_workgroups": limit, "alone_GBps": round(payload / x_med / 1e6, 2),
                "gemm_slowdown_pct": round(100.0 * (with_d - base_d) / base_d, 2)})
        ds.ds_config_set("grid_limit", 0)
    out["gather_into_pinned_host"] = direct
    del host_img

    # (3) Differential snapshot (the paper's future work): keep the previous image in HBM, gather the new
    # one beside it, compare them chunk by chunk on the device, copy only the chunks that changed.
    cb = 32 * MiB                                         # the granularity at which changed data is copied
    n_blocks = -(-total // cb)
    img_a = torch.empty(max(total, 16), dtype=torch.uint8, device=c.dev)
    img_b = torch.empty(max(total, 16), dtype=torch.uint8, device=c.dev)
    flags_dev = torch.zeros(n_blocks, dtype=torch.int32, device=c.dev)
    host_img = torch.empty(max(total, 16), dtype=torch.uint8, pin_memory=True)
    L.arena.copy_(pristine)
    keep = L.arena.clone()
    rows = []
    for frac in (1.0, 0.25, 0.05, 0.0):
        # the reference: image of the unchanged state, on the device and (whole) in host memory
        L.arena.copy_(keep)
        ds.ds_pack(L.plan, img_a.data_ptr(), 0, total, c.stream)
        torch.cuda.synchronize()
        host_img[:total].copy_(img_a[:total])
        n_mut = int(L.arena.numel() * frac)
        if n_mut:
            L.arena[:n_mut].add_(1)                                # this share of the rank's memory changes
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ds.ds_pack(L.plan, img_b.data_ptr(), 0, total, c.stream)
        ds.ds_image_diff(img_a.data_ptr(), img_b.data_ptr(), total, cb, flags_dev.data_ptr(), c.stream)
        dirty = flags_dev.cpu().nonzero().flatten().tolist()       # the one host synchronisation
        for k in dirty:
            lo, hi = k * cb, min((k + 1) * cb, total)
            host_img[lo:hi].copy_(img_b[lo:hi], non_blocking=True)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3
        ok = bool(torch.equal(host_img[:total], img_b[:total].cpu()))   # the host image is the new image
        if frac == 0.0 and L.want is not None:
            ok = ok and same_bytes(c, host_img[:total].numpy(), L.want)  # ... and, unchanged, the oracle's
        rows.append({"share_of_memory_changed": frac, "dirty_chunks": len(dirty), "chunks": n_blocks,
                     "ms": round(ms, 3), "effective_GBps": round(payload / ms / 1e6, 1),
                     "host_image_equals_new_image": ok})
    L.arena.copy_(keep)
    out["differential_snapshot"] = {
        "rows": rows,
        "note": "gather + device compare of two images (ds_image_diff, one flag per 32 MiB chunk) + "
                "copies of the changed chunks only; costs a second image in HBM and one host synchronisation"}
    del img_a, img_b, host_img

    # (4) Compressed snapshot (the other data reduction the paper's conclusions name): block elision.  Gather,
    # find the blocks whose 16-byte units are all equal, pack the others densely, copy only those (plus one
    # pattern and one flag per block).  Measured on the state as it is (normally distributed values: nothing
    # to elide) and with the two Adam moment partitions zeroed, as they are right after initialisation.
    from_oracle = None
    if L.want is not None:
        from oracle import image_compress as ic
        from_oracle = ic
    block = 64 << 10
    n_blk = -(-total // block)
    img = torch.empty(max(total, 16), dtype=torch.uint8, device=c.dev)
    packed = torch.empty(n_blk * block, dtype=torch.uint8, device=c.dev)
    keep_d = torch.zeros(n_blk, dtype=torch.int32, device=c.dev)
    pos_d = torch.zeros(n_blk + 1, dtype=torch.int32, device=c.dev)
    pats_d = torch.zeros(n_blk * 16, dtype=torch.uint8, device=c.dev)
    host_packed = torch.empty(n_blk * block, dtype=torch.uint8, pin_memory=True)
    host_pats = torch.empty(n_blk * 16, dtype=torch.uint8, pin_memory=True)
    rows = []
    flats = [sh for sh in L.w.shards if sh.dtype == "f32" and len(sh.shape) == 1]
    flats = sorted(flats, key=lambda sh: -sh.nbytes)[:3]
    for label, zeroed in (("state as it is", []), ("Adam moments zeroed", flats[1:])):
        L.arena.copy_(keep)
        for sh in zeroed:
            L.arena[sh.byte_offset:sh.byte_offset + sh.nbytes].zero_()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ds.ds_pack(L.plan, img.data_ptr(), 0, total, c.stream)
        ds.ds_image_compress(img.data_ptr(), total, block, keep_d.data_ptr(), pos_d.data_ptr(), pats_d.data_ptr(),
                             packed.data_ptr(), c.stream)
        pos_h = pos_d.cpu()                                        # the one host synchronisation
        n_kept = int(pos_h[-1])
        t_kernels = (time.perf_counter() - t0) * 1e3
        host_packed[:n_kept * block].copy_(packed[:n_kept * block], non_blocking=True)
        host_pats.copy_(pats_d, non_blocking=True)
        keep_h = keep_d.cpu()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3
        exact = None
        if from_oracle is not None:
            np = c.np
            back = from_oracle.decompress(keep_h.numpy().astype(np.uint32), pos_h.numpy().astype(np.uint32),
                                          host_pats.numpy().reshape(-1, 16), host_packed.numpy(), total, block)
            if not zeroed:
                exact = same_bytes(c, back, L.want)               # the oracle's image of the unchanged state
            else:
                exact = same_bytes(c, back, img[:total].cpu().numpy())
        out_bytes = n_kept * block + n_blk * 20
        rows.append({"state": label, "blocks": n_blk, "kept_blocks": n_kept, "bytes_over_the_link": out_bytes,
                     "ratio": round(out_bytes / total, 4), "gather_and_compress_ms": round(t_kernels, 3),
                     "ms": round(ms, 3), "effective_GBps": round(payload / ms / 1e6, 1),
                     "oracle_decompression_gives_the_image": exact})
    L.arena.copy_(keep)
    out["compressed_snapshot"] = {
        "block_bytes": block, "rows": rows,
        "note": "constant 64 KiB blocks are replaced by their 16-byte unit (ds_image_compress); costs a second image "
                "in HBM and one host synchronisation; pays only where the state holds constant regions"}
    del img, packed, host_packed, keep
    return out


def file_cuts(c: Ctx, L: Loaded):
    """The rank's shard table cut into consecutive runs of about equal bytes, one per file."""
    n, payload = L.n, L.payload
    F = min(c.args.files, n)
    cuts, acc, sizes = [0], 0, [c.ds.ds_plan_shard(L.plan, i)[3] for i in range(n)]
    for i in range(n):
        acc += sizes[i]
        if acc >= payload * len(cuts) / F and len(cuts) < F and i + 1 < n:
            cuts.append(i + 1)
    cuts.append(n)
    return cuts


def rank_files_leg(c: Ctx, L: Loaded, cfg, d):
    """One plan over all files of the rank (Sec. VI-D: a 7B rank writes 20): ONE snapshot, its chunks cut at the
    files' boundaries by the flush, one checkpoint writer per file; beside it the same state as one file through
    the same engine.  Files are consecutive runs of the table, so the files' tensor regions one behind the other
    are the single image, which is what the parity leg's oracle image is compared with."""
    ds, torch, np, args = c.ds, c.torch, c.np, c.args
    cuts = file_cuts(c, L)
    F = len(cuts) - 1
    file_of = [f for f in range(F) for _ in range(cuts[f + 1] - cuts[f])]
    descs = ds.make_descs(L.w.shards, L.arena.data_ptr())
    regions, total = ds.ds_layout_assign_files(descs, file_of, L.n, F, L.w.align)
    assert total == L.total
    t0 = time.perf_counter()
    plan = ds.ds_plan_create_files(descs, file_of, L.n, F, L.w.align, ds.DS_PLAN_STRICT)
    plan_ms = (time.perf_counter() - t0) * 1e3
    eng = c.engine(cfg, flags=0)
    file_flags = ds.DS_FILE_DIRECT | (ds.DS_FILE_URING if args.file_engine == "uring" else 0)
    paths = [os.path.join(d, f"ds_bench_{os.getpid()}_part{f}.ckpt") for f in range(F)]
    one = os.path.join(d, f"ds_bench_{os.getpid()}_whole.ckpt")
    res = {"workload": L.name, "dir": d, "files": F, "smallest_region_bytes": min(regions),
           "largest_region_bytes": max(regions), "threads": args.file_threads, "d2h_chunk_bytes": cfg["chunk"],
           "stage_slot_bytes": cfg["slot"], "stage_slots": cfg["slots"], "plan_create_ms": round(plan_ms, 3)}
    try:
        best = None                                      # one warm-up, then the better of two timed attempts
        for attempt in ("warm-up", "timed", "timed"):
            for path in paths:                           # new files every time: truncating the warm-up's would
                if os.path.exists(path):                 # be charged to the request
                    os.remove(path)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ev = ds.ds_snapshot_async(eng, plan, c.stream)
            parts = [ds.ds_ckpt_create_part(paths[f], plan, f, file_flags) for f in range(F)]
            ds.ds_ckpt_flush_snapshot_parts(parts, ev, args.file_threads)
            ds.ds_event_wait_on_stream(ev, c.stream)
            ds.ds_event_wait_captured(ev)
            cap_ms = (time.perf_counter() - t0) * 1e3    # request -> every tensor of every file may be mutated
            nbytes = sum(ds.ds_ckpt_finish(ck)[0] for ck in parts)
            files_s = time.perf_counter() - t0
            ds.ds_event_wait(ev)
            st = ds.ds_event_stats(ev)
            ds.ds_event_destroy(ev)
            if attempt == "timed" and (best is None or cap_ms < best[0]):
                best = (cap_ms, st, files_s)
        cap_ms, st, files_s = best
        res.update({"file_bytes": nbytes, "request_to_all_captured_ms": round(cap_ms, 3),
                    "capture_ms_device_events": round(st["capture_ms"], 3),
                    "gather_launches": st["n_pack_launches"],
                    "snapshot_to_files_GBps": round(nbytes / files_s / 1e9, 2)})
        if L.want is not None:
            at, same = 0, True
            for f in range(F):
                got = np.fromfile(paths[f], dtype=np.uint8, count=regions[f])
                same = same and got.size == regions[f] and same_bytes(c, got, L.want[at:at + regions[f]])
                at += regions[f]
            res["tensor_regions_byte_exact_vs_oracle"] = bool(same)
        # all files back into the GPU in one restore
        t0 = time.perf_counter()
        readers = [ds.ds_ckpt_open(p) for p in paths]
        rev = ds.ds_ckpt_restore_parts(readers, eng, plan, args.file_threads, ds.DS_FILE_DIRECT, c.stream)
        ds.ds_event_wait(rev)
        load_s = time.perf_counter() - t0
        ds.ds_event_destroy(rev)
        for r in readers:
            ds.ds_ckpt_close(r)
        res["files_to_gpu_GBps"] = round(L.payload / load_s / 1e9, 2)
        # the same state as ONE file, same engine, the better of two attempts
        best = None
        for attempt in ("timed", "timed"):
            if os.path.exists(one):
                os.remove(one)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ev = ds.ds_snapshot_async(eng, L.plan, c.stream)
            ck = ds.ds_ckpt_create(one, L.plan, file_flags)
            ds.ds_ckpt_flush_snapshot(ck, ev, args.file_threads)
            ds.ds_event_wait_on_stream(ev, c.stream)
            ds.ds_event_wait_captured(ev)
            cap1_ms = (time.perf_counter() - t0) * 1e3
            nbytes1, _ = ds.ds_ckpt_finish(ck)
            one_s = time.perf_counter() - t0
            ds.ds_event_wait(ev)
            st1 = ds.ds_event_stats(ev)
            ds.ds_event_destroy(ev)
            if best is None or cap1_ms < best[0]:
                best = (cap1_ms, st1, one_s)
        cap1_ms, st1, one_s = best
        res["same_state_as_one_file"] = {"request_to_captured_ms": round(cap1_ms, 3),
                                         "capture_ms_device_events": round(st1["capture_ms"], 3),
                                         "snapshot_to_file_GBps": round(nbytes1 / one_s / 1e9, 2)}
    except ds.DsError as e:
        res["error"] = str(e)
    finally:
        ds.ds_engine_destroy(eng)
        torch.cuda.synchronize()
        ds.ds_plan_destroy(plan)
        for path in paths + [one]:
            if os.path.exists(path):
                os.remove(path)
    log(f"[bench] {L.name} as {F} files through one plan: {res.get('snapshot_to_files_GBps')} GB/s to {d}, "
        f"request -> all captured {res.get('request_to_all_captured_ms')} ms "
        f"(one file: {res.get('same_state_as_one_file', {}).get('request_to_captured_ms')} ms)")
    return res


def several_plans(c: Ctx, L: Loaded, cfg):
    """One rank's checkpoint split over several files (the paper's 7B rank writes 20, Sec. VI-D): one plan per
    file over consecutive shards of about equal bytes, all through the one engine, back to back."""
    ds, torch, args = c.ds, c.torch, c.args
    n, payload = L.n, L.payload
    cuts = file_cuts(c, L)
    plans = []
    for a, b in zip(cuts[:-1], cuts[1:]):
        dg = ds.make_descs(L.w.shards[a:b], L.arena.data_ptr())
        ds.ds_layout_assign(dg, b - a, L.w.align)
        plans.append(ds.ds_plan_create(dg, b - a, L.w.align, ds.DS_PLAN_STRICT))
    eng = c.engine(cfg)

    def several():
        t0 = time.perf_counter()
        evs = [ds.ds_snapshot_async(eng, pl, c.stream) for pl in plans]
        ds.ds_event_wait_on_stream(evs[-1], c.stream)      # snapshots run in order: the last gate covers all
        ds.ds_event_wait_captured(evs[-1])
        t_cap = time.perf_counter() - t0                 # first request -> every tensor may be mutated (host clock)
        for ev in evs:
            ds.ds_event_wait(ev)
        return evs, t_cap, time.perf_counter() - t0
    try:
        for ev in several()[0]:
            ds.ds_event_destroy(ev)
        torch.cuda.synchronize()
        evs, cap_s, several_s = several()
        for ev in evs:
            ds.ds_event_destroy(ev)
    finally:
        ds.ds_engine_destroy(eng)
    res = {"plans": len(plans), "smallest_image_bytes": min(ds.ds_plan_info(pl)["total_bytes"] for pl in plans),
           "largest_image_bytes": max(ds.ds_plan_info(pl)["total_bytes"] for pl in plans),
           "GBps_into_host_ring": round(payload / several_s / 1e9, 2),
           "first_request_to_all_captured_ms": round(cap_s * 1e3, 3),
           "note": "the same bytes as one image, requested as one snapshot per file; compare with `value`"}
    return res, plans


def restore_leg(c: Ctx, L: Loaded, cfg):
    """Restore pipeline rate with a null producer (slots submitted as they are: the link and the scatter)."""
    ds, torch = c.ds, c.torch
    eng = c.engine(cfg)
    try:
        for _ in range(2):                               # one warm-up (new staging is slow on first touch), one timed
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            rev = ds.ds_restore_begin(eng, L.plan, c.stream)
            while True:
                slot = ds.ds_restore_next_slot(rev)
                if slot is None:
                    break
                ds.ds_restore_submit(rev, slot[0])
            ds.ds_event_wait(rev)
            restore_s = time.perf_counter() - t0
            rst = ds.ds_event_stats(rev)
            ds.ds_event_destroy(rev)
    finally:
        ds.ds_engine_destroy(eng)
    return {"GBps_null_producer": round(L.payload / restore_s / 1e9, 2), "ms": round(restore_s * 1e3, 3),
            "h2d_link_peak_measured_GBps": round(c.link_h2d, 2),
            "frac_of_h2d_peak": round(L.payload / restore_s / 1e9 / c.link_h2d, 4),
            "scatter_ms": round(rst["pack_ms"], 3), "scatter_launches": rst["n_pack_launches"]}


def file_leg(c: Ctx, L: Loaded, cfg, file_plans):
    """The checkpoint file: snapshot -> ring -> tensor region (writer threads) with an object log appended
    behind it at the same time, trailer last; then file -> ring -> GPU."""
    import threading
    ds, torch, args = c.ds, c.torch, c.args
    plan, payload = L.plan, L.payload
    eng2 = c.engine(cfg, flags=0)
    obj_chunk = os.urandom(64 << 10)
    n_obj_threads, chunks_per_thread = 2, 128             # 16 MiB of serialized objects in 64 KiB chunks
    file_flags = ds.DS_FILE_DIRECT | (ds.DS_FILE_URING if args.file_engine == "uring" else 0)

    def one_dir(d):
        path = os.path.join(d, f"ds_bench_{os.getpid()}.ckpt")
        try:
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ev = ds.ds_snapshot_async(eng2, plan, c.stream)
            ck = ds.ds_ckpt_create(path, plan, file_flags)
            ds.ds_ckpt_flush_snapshot(ck, ev, args.file_threads)

            def objects(t):
                for k in range(chunks_per_thread):
                    ds.ds_ckpt_append(ck, 1000 + t * 16 + k % 16, obj_chunk)
            ts = [threading.Thread(target=objects, args=(t,)) for t in range(n_obj_threads)]
            for t in ts:
                t.start()
            ds.ds_event_wait_on_stream(ev, c.stream)
            for t in ts:
                t.join()
            nbytes, _ = ds.ds_ckpt_finish(ck)
            flush_s = time.perf_counter() - t0
            ds.ds_event_wait(ev)
            fst = ds.ds_event_stats(ev)
            ds.ds_event_destroy(ev)
            t0 = time.perf_counter()
            rd = ds.ds_ckpt_open(path)
            rev = ds.ds_ckpt_restore(rd, eng2, plan, args.file_threads, ds.DS_FILE_DIRECT, c.stream)
            ds.ds_event_wait(rev)
            load_s = time.perf_counter() - t0
            ds.ds_event_destroy(rev)
            lay = ds.ds_ckpt_layout_info(rd)
            ds.ds_ckpt_close(rd)
            return {"dir": d, "file_bytes": nbytes, "object_log_bytes": lay["log_end"] - lay["tensor_bytes"],
                    "object_chunks": lay["n_chunks"],
                    "snapshot_to_file_GBps": round(nbytes / flush_s / 1e9, 2),
                    "capture_ms": round(fst["capture_ms"], 3),   # tensors free again, whatever the storage does
                    "image_in_host_ring_ms": round(fst["total_ms"], 3),
                    "file_to_gpu_GBps": round(payload / load_s / 1e9, 2)}
        except ds.DsError as e:
            return {"dir": d, "error": str(e)}
        finally:
            if os.path.exists(path):
                os.remove(path)

    try:
        dirs = [args.file_dir] + (["/dev/shm"] if os.path.isdir("/dev/shm") and args.file_dir != "/dev/shm" else [])
        file_tier = {"threads": args.file_threads, "engine": args.file_engine, "d2h_chunk_bytes": cfg["chunk"],
                     "io_uring_available": ds.ds_config_get("io_uring_available"),
                     "note": "request -> trailer written (page cache, no fsync); open + check -> tensors restored; "
                             "/dev/shm is memory-backed: the software path without the disk",
                     "runs": [one_dir(d) for d in dirs]}
        if file_plans:
            # the same split, each plan into a checkpoint file of its own, all flushes in flight at once
            paths = [os.path.join(dirs[0], f"ds_bench_{os.getpid()}_{k}.ckpt") for k in range(len(file_plans))]
            try:
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                evs, cks = [], []
                for pl, path in zip(file_plans, paths):
                    ev = ds.ds_snapshot_async(eng2, pl, c.stream)
                    ck = ds.ds_ckpt_create(path, pl, file_flags)
                    ds.ds_ckpt_flush_snapshot(ck, ev, max(1, args.file_threads // 2))
                    evs.append(ev)
                    cks.append(ck)
                ds.ds_event_wait_on_stream(evs[-1], c.stream)
                ds.ds_event_wait_captured(evs[-1])
                cap_ms = (time.perf_counter() - t0) * 1e3   # first request -> every tensor may be mutated
                nbytes = sum(ds.ds_ckpt_finish(ck)[0] for ck in cks)
                files_s = time.perf_counter() - t0
                for ev in evs:
                    ds.ds_event_wait(ev)
                    ds.ds_event_destroy(ev)
                file_tier["several_files"] = {"dir": dirs[0], "files": len(paths), "file_bytes": nbytes,
                                              "threads_per_file": max(1, args.file_threads // 2),
                                              "first_request_to_all_captured_ms": round(cap_ms, 3),
                                              "snapshot_to_files_GBps": round(nbytes / files_s / 1e9, 2)}
            except ds.DsError as e:
                file_tier["several_files"] = {"error": str(e)}
            finally:
                for path in paths:
                    if os.path.exists(path):
                        os.remove(path)
    finally:
        ds.ds_engine_destroy(eng2)
    return file_tier


def timeline_leg(c: Ctx, L: Loaded, cfg):
    """The timeline of one snapshot, tier by tier, written as text."""
    ds, args = c.ds, c.args
    eng_t = c.engine(cfg, flags=ds.DS_ENGINE_AUTO_RELEASE | ds.DS_ENGINE_TRACE)
    for _ in range(2):                                   # the second one is reported
        ev = ds.ds_snapshot_async(eng_t, L.plan, c.stream)
        ds.ds_event_wait(ev)
        recs = ds.ds_event_trace(ev)
        tst = ds.ds_event_stats(ev)
        ds.ds_event_destroy(ev)
    ds.ds_engine_destroy(eng_t)
    gat = [r for r in recs if r["kind"] == 0]
    cop = [r for r in recs if r["kind"] == 1]
    busy, cur_b, cur_e = 0.0, None, None                 # union of the copy intervals = time the link works
    for r in sorted(cop, key=lambda r: r["begin_ms"]):
        if cur_e is None or r["begin_ms"] > cur_e:
            busy += (cur_e - cur_b) if cur_e is not None else 0.0
            cur_b, cur_e = r["begin_ms"], r["end_ms"]
        else:
            cur_e = max(cur_e, r["end_ms"])
    busy += (cur_e - cur_b) if cur_e is not None else 0.0
    lines = [f"# Timeline of one snapshot, workload {L.name} (device clock, ms since the request)", "",
             "Command:", "",
             "    python3 bench.py " + " ".join(a for a in sys.argv[1:]), "",
             f"image {L.total} B; ring slot / copy {cfg['chunk']} B; staging {cfg['slots']} x "
             f"{cfg['slot']} B; copy streams {cfg['copy_streams']}", "",
             "| step | image range | begin ms | end ms | duration ms | rate |", "|---|---|---|---|---|---|"]
    for r in gat:
        d = r["end_ms"] - r["begin_ms"]
        lines.append(f"| gather launch {r['index']} | [{r['file_off']}, {r['file_off'] + r['len']}) | {r['begin_ms']:.3f} | "
                     f"{r['end_ms']:.3f} | {d:.3f} | {2 * r['len'] / d / 1e6:.0f} GB/s read+write |")
    show = cop if len(cop) <= 8 else cop[:4] + [None] + cop[-3:]
    for r in show:
        if r is None:
            lines.append("| ... | | | | | |")
            continue
        d = r["end_ms"] - r["begin_ms"]
        lines.append(f"| copy of chunk {r['index']} | [{r['file_off']}, {r['file_off'] + r['len']}) | {r['begin_ms']:.3f} | "
                     f"{r['end_ms']:.3f} | {d:.3f} | {r['len'] / d / 1e6:.1f} GB/s |")
    if cop:
        durs = sorted(r["end_ms"] - r["begin_ms"] for r in cop)
        first, last = min(r["begin_ms"] for r in cop), max(r["end_ms"] for r in cop)
        lines += ["", f"{len(cop)} copies: median duration {durs[len(durs) // 2]:.3f} ms; first copy starts at "
                  f"{first:.3f} ms ({first - gat[0]['end_ms']:.3f} ms after the first gather ended), last one ends at "
                  f"{last:.3f} ms; the link is busy {busy:.3f} ms of the {last - first:.3f} ms between them "
                  f"({100 * busy / (last - first):.1f} %); the tensors are free again at {tst['capture_ms']:.3f} ms, "
                  f"the image is in the host ring at {tst['total_ms']:.3f} ms = {L.payload / tst['total_ms'] / 1e6:.2f} GB/s."]
    with open(args.timeline, "w") as f:
        f.write("\n".join(lines) + "\n")
    log(f"[bench] timeline written to {args.timeline}")


def microbench(c: Ctx) -> int:
    """Gather / scatter rates (read+write GB/s of payload, median of the timed launches) on tables made to
    isolate one path of the kernel: (a) contiguous u8 tensors of one size each at 512-byte alignment, so that
    every 16 KiB chunk holds tile boundaries and takes the general path; (b) one 2-D u8 view per (row, pitch)
    pair, which takes the lean row path.  The plain copy probe over the same number of bytes is the ceiling.
    The parent buffer is 16 GiB, so that views at large pitches still gather hundreds of megabytes (a table of a
    few dozen megabytes would sit in the 256 MB of last-level cache and measure that)."""
    ds, torch, args = c.ds, c.torch, c.args
    stream = c.stream
    ds.ds_config_set("variant", args.variant)
    BUF = 16 << 30
    buf = torch.empty(BUF, dtype=torch.uint8, device=c.dev)
    buf[:3 << 30].random_(0, 255)
    reps = max(1, args.reps)

    def timed(fn):
        return c.timed(fn, reps=reps, warm=min(3, reps))[0]

    def run(tensors, align):
        descs = ds.make_descs_from_tensors(tensors)
        n = len(tensors)
        total = ds.ds_layout_assign(descs, n, align)
        plan = ds.ds_plan_create(descs, n, align, 0)
        info = ds.ds_plan_info(plan)
        img = torch.empty(total, dtype=torch.uint8, device=c.dev)
        other = torch.empty(total, dtype=torch.uint8, device=c.dev)
        p = timed(lambda: ds.ds_pack(plan, img.data_ptr(), 0, total, stream))
        u = timed(lambda: ds.ds_unpack(plan, img.data_ptr(), 0, total, stream))
        cp = timed(lambda: ds.ds_copy_probe(other.data_ptr(), img.data_ptr(), total & ~15, stream))
        ds.ds_plan_destroy(plan)
        pay = info["payload_bytes"]
        return {"payload_bytes": pay, "image_bytes": total, "chunks": info["n_chunks"],
                "general_chunks": info["n_general_chunks"], "gather_GBps": round(2 * pay / p / 1e6),
                "scatter_GBps": round(2 * pay / u / 1e6), "copy_probe_GBps": round(2 * (total & ~15) / cp / 1e6),
                # the gather also writes the padding: bytes it really moves (payload read + image written)
                "gather_moved_GBps": round((pay + total) / p / 1e6)}

    out = {"microbench": True, "unit": "GB/s read+write of payload", "variant": args.variant, "general_path": [],
           "row_path": []}
    # --tables general:200,rows:5504x22016 limits the run to those tables (for counter runs, with --reps)
    want = set(args.tables.split(",")) if args.tables else None
    if want is None or "contiguous" in want:
        out["contiguous_1GiB"] = run([buf[:1 << 30]], 4096)
    sizes = [12288, 12296, 1024, 1032, 208, 200]
    shapes = [(2048, 2304), (2048, 4096), (2048, 8192), (2048, 8256), (2048, 16384), (2048, 65536), (2048, 131072),
              (5504, 22016), (5504, 22528), (5504, 7552), (2752, 11008), (2752, 11264), (512, 2048)]
    for item in sorted(want or ()):                      # tables beyond the standard ones may be named too
        kind, _, spec = item.partition(":")
        if kind == "general" and int(spec) not in sizes:
            sizes.append(int(spec))
        if kind == "rows" and tuple(map(int, spec.split("x"))) not in shapes:
            shapes.append(tuple(map(int, spec.split("x"))))
    for size in sizes:
        if want is not None and f"general:{size}" not in want:
            continue
        pitch = (size + 511) // 512 * 512 + 512
        n = (1 << 30) // pitch
        r = run([buf[i * pitch + 3: i * pitch + 3 + size] for i in range(n)], 512)
        out["general_path"].append({"tensor_bytes": size, "tensors": n, **r})
        log(f"[microbench] general path, tensors of {size} B: {r['gather_GBps']} / {r['scatter_GBps']} GB/s")
    for row, pitch in shapes:
        if want is not None and f"rows:{row}x{pitch}" not in want:
            continue
        rows = min((768 << 20) // row, (BUF - row) // pitch)
        r = run([torch.as_strided(buf, (rows, row), (pitch, 1))], 4096)
        out["row_path"].append({"row_bytes": row, "pitch_bytes": pitch, "rows": rows, **r})
        log(f"[microbench] rows of {row} B at pitch {pitch} B: {r['gather_GBps']} / {r['scatter_GBps']} GB/s "
            f"(copy probe {r['copy_probe_GBps']})")
    print(json.dumps(out), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama7b", choices=list(WORKLOADS),
                    help="the headline workload (the top-level fields of the JSON line)")
    ap.add_argument("--only", action="store_true", help="measure the headline workload only (no per_workload list "
                                                        "of the other shard sets, no cap-binding runs)")
    ap.add_argument("--ring-bytes", type=int, default=2 * GiB, help="pinned host ring (configs[4] caps it at 2 GiB)")
    ap.add_argument("--chunk-bytes", type=int, default=128 * MiB, help="one device-to-host copy / ring slot")
    ap.add_argument("--stage-slot-bytes", type=int, default=2 * GiB, help="device staging slot = bytes per gather launch")
    ap.add_argument("--stage-slots", type=int, default=2)
    ap.add_argument("--copy-streams", type=int, default=1)
    ap.add_argument("--first-launch-bytes", type=int, default=0, help="short first gather launch (0 = none)")
    ap.add_argument("--no-overlap", action="store_true", help="skip the concurrent-GEMM leg (configs[4])")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle: no parity, no CPU baseline")
    ap.add_argument("--no-file", action="store_true", help="skip the file-tier leg")
    ap.add_argument("--no-experiments", action="store_true", help="skip the capture variants")
    ap.add_argument("--file-dir", default="/tmp", help="where the file-tier leg writes its image")
    ap.add_argument("--file-threads", type=int, default=8)
    ap.add_argument("--manifest", default=None, metavar="FILE",
                    help="where the headline run's input manifest goes (seed, shard table, realised sizes and "
                         "offsets); default bench_out/manifest_<workload>.json, '-' = none")
    ap.add_argument("--files", type=int, default=20, help="--experiments: files the rank's state is split over")
    ap.add_argument("--file-engine", default="threads", choices=["threads", "uring"],
                    help="writers of the file tier: pwrite threads, or one thread with that many writes in flight "
                         "through io_uring")
    ap.add_argument("--gemm-iters", type=int, default=20, help="iterations of the overlap leg")
    ap.add_argument("--experiments", action="store_true",
                    help="the capture variants in full (more grid limits, the rank's state as several plans and "
                         "several checkpoint files); the default run measures a compact set of them")
    ap.add_argument("--variant", type=int, default=0, choices=[0, 1, 2, 3, 4, 5],
                    help="kernel variant (ds_config_set): 0 default, 1 plain accesses, 2 non-temporal global accesses, "
                         "3 default accesses with work-group i on chunk i, 4 no aligned-load route, "
                         "5 four wavefronts per SIMD also for plans of mostly general chunks")
    ap.add_argument("--timeline", default=None, metavar="FILE",
                    help="also trace one snapshot step by step (gather launches, every chunk copy) and write the "
                         "timeline to FILE as text")
    ap.add_argument("--timed-only", action="store_true",
                    help="stop after the timed region (so that a kernel trace holds the timed launches only)")
    ap.add_argument("--kernels-only", action="store_true",
                    help="only gather, scatter and the copy probe, 5 launches each (for counter runs)")
    ap.add_argument("--microbench", action="store_true",
                    help="instead of the workload: gather and scatter rates on synthetic tables that isolate one path of "
                         "the kernel each (every chunk general with tensors of one size; one 2-D view per row length "
                         "and pitch), one JSON object")
    ap.add_argument("--tables", default=None,
                    help="--microbench: only these tables, e.g. contiguous,general:200,rows:5504x22016")
    ap.add_argument("--reps", type=int, default=15, help="--microbench: timed launches per kernel and table")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build is the one-GPU hot path; it has no multi-GPU leg (run with --gpus 1).")
        return 2

    c = Ctx(args)
    ds, torch = c.ds, c.torch
    if args.microbench:
        return microbench(c)
    props = torch.cuda.get_device_properties(c.dev)
    ds.ds_config_set("variant", args.variant)
    cfg = engine_cfg(args)

    L = Loaded(c, args.workload)
    manifest = write_manifest(c, L)

    if args.kernels_only:
        image_dev = torch.empty(max(L.total, 16), dtype=torch.uint8, device=c.dev)
        copy_src = torch.empty_like(image_dev)
        for _ in range(5):
            ds.ds_pack(L.plan, image_dev.data_ptr(), 0, L.total, c.stream)
        for _ in range(5):
            ds.ds_copy_probe(image_dev.data_ptr(), copy_src.data_ptr(), L.total & ~15, c.stream)
        for _ in range(5):
            ds.ds_unpack(L.plan, image_dev.data_ptr(), 0, L.total, c.stream)
        torch.cuda.synchronize()
        print(json.dumps({"kernels_only": True, "workload": args.workload, "image_bytes": L.total,
                          "payload_bytes": L.payload, "copy_probe_bytes": L.total & ~15,
                          "kernel_source_digest": ds.kernel_source_digest()}), flush=True)
        L.close(c)
        return 0

    measure_link(c)

    if args.timed_only:
        tr = timed_region(c, L, cfg, args.steps, args.warmup, extras=False)
        print(json.dumps({"metric": METRIC, "value": tr["value"], "unit": "GB/s", "steps": args.steps,
                          "warmup": args.warmup, "ms_per_step": tr["ms_per_step"], "workload": args.workload,
                          "timed_only": True, "roofline": tr["roofline"]}), flush=True)
        L.close(c)
        return 0

    # ---- the headline workload: timed region, standalone kernels, parity, CPU baseline -----------------
    head, tr, cpu_baseline = workload_entry(c, L, cfg, args.steps, args.warmup, want_baseline=True)
    if args.timeline:
        timeline_leg(c, L, cfg)
    restore = restore_leg(c, L, cfg)
    L.arena.copy_(torch.from_numpy(L.w.arena))           # the null producer has scattered whatever the ring held

    cap_binding = []
    if not args.only and args.workload == "llama7b":
        # the 7B image (1.43 GiB) fits the 2 GiB ring: a ring of 512 MiB makes the cap bind
        cap_binding.append(cap_binding_run(c, L, engine_cfg(args, ring=512 * MiB), min(args.steps, 10),
                                           "host ring smaller than the image"))
        cap_binding.append(cap_binding_run(c, L, engine_cfg(args, ring=512 * MiB, slot=512 * MiB, slots=1),
                                           min(args.steps, 10), "host ring and device staging smaller than the image"))

    overlap, experiments = None, {}
    loop = gemm = ohead = oeng = None
    if not args.no_overlap:
        overlap, loop, gemm, ohead, oeng = overlap_leg(c, L, cfg, tr["one_total_ms"])
        L.arena.copy_(torch.from_numpy(L.w.arena))       # the loop has mutated the tensors
    try:
        if not args.no_experiments:
            experiments = experiments_leg(c, L, cfg, loop, gemm, ohead, args.experiments)
    finally:
        if oeng is not None:
            ds.ds_engine_destroy(oeng)
    del loop, gemm
    file_plans = []
    if args.experiments:
        experiments["rank_state_as_several_plans"], file_plans = several_plans(c, L, cfg)
    # the flush consumer gets finer ring slots than the null consumer of the timed region: more writes in flight
    file_chunk = min(args.chunk_bytes, 32 * MiB)
    file_tier = None if args.no_file else file_leg(c, L, engine_cfg(args, chunk=file_chunk), file_plans)
    if file_tier is not None:
        file_tier["one_plan_of_files"] = [rank_files_leg(c, L, engine_cfg(args, chunk=file_chunk), args.file_dir)]
    torch.cuda.synchronize()
    for pl in file_plans:
        ds.ds_plan_destroy(pl)
    L.close(c)
    settle(c)

    # ---- the other shard sets: the same measurement and the same parity check, each in this run --------
    per_workload = []
    if not args.only:
        k_steps, k_warm = min(args.steps, 10), min(args.warmup, 3)
        for name in WORKLOADS:
            if name == args.workload:
                per_workload.append(dict(head))
                continue
            Lx = Loaded(c, name)
            try:
                # staging as large as the image where it does not fit the default 2 x 2 GiB (288 GB of HBM make
                # that an ordinary setting); the default staging on the same state is under cap_binding
                cfgx = cfg if Lx.total <= cfg["slot"] else engine_cfg(args, slot=8 * GiB, slots=1)
                entry, _, _ = workload_entry(c, Lx, cfgx, k_steps, k_warm)
                per_workload.append(entry)
                if Lx.total > cfg["slot"] and name == "llama70b":
                    cap_binding.append(cap_binding_run(c, Lx, cfg, min(k_steps, 5),
                                                       "host ring and device staging smaller than the image"))
                if name == "llama70b" and file_tier is not None:
                    # staging as large as the image: every gate opens behind the gathers alone
                    file_tier["one_plan_of_files"].append(rank_files_leg(
                        c, Lx, engine_cfg(args, chunk=file_chunk, slot=8 * GiB, slots=1), args.file_dir))
            finally:
                Lx.close(c)
                del Lx
                settle(c)

    parities = [e["parity"] for e in per_workload] or [head["parity"]]
    out = {
        "metric": METRIC,
        "value": head["value"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {
            "workload": head["workload"], "payload_bytes": head["payload_bytes"],
            "image_bytes": head["image_bytes"], "shards": head["shards"], "align": head["align"],
            **engine_json(cfg), "workgroup_chunk_bytes": 16384, "manifest": manifest,
        },
        "roofline": head["roofline"],
        "cpu_baseline": cpu_baseline,
        "parity": head["parity"],
        "d2h": head["d2h"],
        "snapshot_latency_ms": head["snapshot_latency_ms"],
        "pipelined_GBps": head["pipelined_GBps"],
        "capture_ms": head["capture_ms"],
        "submit_host_ms": head["submit_host_ms"],
        "plan_create_ms": head["plan_create_ms"],
        "standalone": head["standalone"],
        "restore": restore,
        "overlap": overlap,
        "per_workload": per_workload,
        "cap_binding": cap_binding,
        "file_tier": file_tier,
        **({"experiments": experiments} if experiments else {}),
        "device": {"name": props.name, "compute_units": props.multi_processor_count,
                   "hbm_bytes": props.total_memory},
        "hip_runtime": ds.hip_runtime_in_use(),
        "kernel_source_digest": ds.kernel_source_digest(),
    }
    print(json.dumps(out), flush=True)
    bad = any("MISMATCH" in p for p in parities) or any(r.get("image_through_consumer_byte_exact_vs_oracle") is False
                                                       for r in cap_binding)
    return 1 if bad else 0


if __name__ == "__main__":
    sys.exit(main())
