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

Prints ONE JSON line.  `value` is payload GB/s of the whole step (link-bound);
`roofline` is the gather kernel against the HBM peak, timed with HIP events on
the stream it runs on; `cpu_baseline` is the CPU oracle's pack of the same
workload on this machine's host cores.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
MiB = 1 << 20
GiB = 1 << 30

WORKLOADS = {
    "tiny_gpt": "configs[0] tiny GPT-style state, 118 shards",
    "llama7b": "configs[1] Llama-7B rank (TP=4, PP=4, ZeRO-1 DP=8), 76 shards",
    "fragmentation": "configs[2] fragmentation stress, 20000 shards",
    "llama70b": "configs[3] Llama-2-70B rank (TP=8, PP=4, ZeRO-1 DP=8), 184 shards",
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def microbench(ds, torch, dev, args) -> int:
    """Gather / scatter rates (read+write GB/s of payload, median of 15 launches) on tables made to isolate
    one path of the kernel: (a) contiguous u8 tensors of one size each at 512-byte alignment, so that every
    16 KiB chunk holds tile boundaries and takes the general path; (b) one 2-D u8 view per (row, pitch)
    pair, which takes the lean row path.  The plain copy probe over the same number of bytes is the ceiling."""
    stream = torch.cuda.current_stream().cuda_stream
    ds.ds_config_set("variant", args.variant)
    buf = torch.empty(3 << 30, dtype=torch.uint8, device=dev).random_(0, 255)

    reps = max(1, args.reps)

    def timed(fn):
        for _ in range(min(3, reps)):
            fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            ts.append((a, b))
        torch.cuda.synchronize()
        return sorted(x.elapsed_time(y) for x, y in ts)[len(ts) // 2]

    def run(tensors, align):
        descs = ds.make_descs_from_tensors(tensors)
        n = len(tensors)
        total = ds.ds_layout_assign(descs, n, align)
        plan = ds.ds_plan_create(descs, n, align, 0)
        info = ds.ds_plan_info(plan)
        img = torch.empty(total, dtype=torch.uint8, device=dev)
        other = torch.empty(total, dtype=torch.uint8, device=dev)
        p = timed(lambda: ds.ds_pack(plan, img.data_ptr(), 0, total, stream))
        u = timed(lambda: ds.ds_unpack(plan, img.data_ptr(), 0, total, stream))
        c = timed(lambda: ds.ds_copy_probe(other.data_ptr(), img.data_ptr(), total & ~15, stream))
        ds.ds_plan_destroy(plan)
        pay = info["payload_bytes"]
        return {"payload_bytes": pay, "image_bytes": total, "chunks": info["n_chunks"],
                "general_chunks": info["n_general_chunks"], "gather_GBps": round(2 * pay / p / 1e6),
                "scatter_GBps": round(2 * pay / u / 1e6), "copy_probe_GBps": round(2 * (total & ~15) / c / 1e6)}

    out = {"microbench": True, "unit": "GB/s read+write of payload", "variant": args.variant, "general_path": [],
           "row_path": []}
    # --tables general:200,rows:5504x22016 limits the run to those tables (for counter runs, with --reps)
    want = set(args.tables.split(",")) if args.tables else None
    if want is None or "contiguous" in want:
        out["contiguous_1GiB"] = run([buf[:1 << 30]], 4096)
    for size in (12288, 12296, 1024, 1032, 208, 200):
        if want is not None and f"general:{size}" not in want:
            continue
        pitch = (size + 511) // 512 * 512 + 512
        n = (1 << 30) // pitch
        r = run([buf[i * pitch + 3: i * pitch + 3 + size] for i in range(n)], 512)
        out["general_path"].append({"tensor_bytes": size, "tensors": n, **r})
        log(f"[microbench] general path, tensors of {size} B: {r['gather_GBps']} / {r['scatter_GBps']} GB/s")
    for row, pitch in ((2048, 2304), (2048, 4096), (2048, 8192), (2048, 8256), (2048, 16384), (2048, 65536), (2048, 131072),
                       (5504, 22016), (5504, 22528), (5504, 7552), (2752, 11008), (512, 2048)):
        if want is not None and f"rows:{row}x{pitch}" not in want:
            continue
        rows = min((1 << 30) // row, ((3 << 30) - row) // pitch)
        r = run([torch.as_strided(buf, (rows, row), (pitch, 1))], 4096)
        out["row_path"].append({"row_bytes": row, "pitch_bytes": pitch, "rows": rows, **r})
        log(f"[microbench] rows of {row} B at pitch {pitch} B: {r['gather_GBps']} / {r['scatter_GBps']} GB/s")
    print(json.dumps(out), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama7b", choices=list(WORKLOADS))
    ap.add_argument("--ring-bytes", type=int, default=2 * GiB, help="pinned host ring (configs[4] caps it at 2 GiB)")
    ap.add_argument("--chunk-bytes", type=int, default=32 * MiB, help="one device-to-host copy / ring slot")
    ap.add_argument("--stage-slot-bytes", type=int, default=2 * GiB, help="device staging slot = bytes per gather launch")
    ap.add_argument("--stage-slots", type=int, default=2)
    ap.add_argument("--copy-streams", type=int, default=2)
    ap.add_argument("--first-launch-bytes", type=int, default=0, help="short first gather launch (0 = none)")
    ap.add_argument("--no-overlap", action="store_true", help="skip the concurrent-GEMM leg (configs[4])")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-file", action="store_true", help="skip the file-tier leg")
    ap.add_argument("--file-dir", default="/tmp", help="where the file-tier leg writes its image")
    ap.add_argument("--file-threads", type=int, default=8)
    ap.add_argument("--manifest", default=None, metavar="FILE",
                    help="where the run's input manifest goes (seed, shard table, realised sizes and offsets); "
                         "default bench_out/manifest_<workload>.json, '-' = none")
    ap.add_argument("--files", type=int, default=20, help="--experiments: files the rank's state is split over")
    ap.add_argument("--file-engine", default="threads", choices=["threads", "uring"],
                    help="writers of the file tier: pwrite threads, or one thread with that many writes in flight "
                         "through io_uring")
    ap.add_argument("--gemm-iters", type=int, default=20, help="iterations of the overlap leg")
    ap.add_argument("--experiments", action="store_true",
                    help="also run the capture variants that are measured, not shipped (direct gather into pinned "
                         "host memory; grid-limited gathers under the GEMM stream)")
    ap.add_argument("--variant", type=int, default=0, choices=[0, 1, 2, 3],
                    help="kernel variant (ds_config_set): 0 default, 1 plain accesses, 2 non-temporal global accesses, "
                         "3 default accesses with work-group i on chunk i")
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

    import numpy as np
    import torch

    import paper_2601_16956_amd as ds

    import workloads as W

    assert torch.cuda.is_available(), "needs the MI355X"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.microbench:
        return microbench(ds, torch, dev, args)
    props = torch.cuda.get_device_properties(dev)
    cores = len(os.sched_getaffinity(0))
    cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))

    t0 = time.time()
    w = W.by_name(args.workload, workers=cores)
    log(f"[bench] generated {w.name}: {len(w.shards)} shards, payload {w.payload_bytes / 1e9:.3f} GB, "
        f"arena {w.arena.size / 1e9:.3f} GB in {time.time() - t0:.1f}s")
    arena = torch.from_numpy(w.arena).to(dev)
    n = len(w.shards)
    descs = ds.make_descs(w.shards, arena.data_ptr())
    total = ds.ds_layout_assign(descs, n, w.align)
    t0 = time.perf_counter()
    plan = ds.ds_plan_create(descs, n, w.align, ds.DS_PLAN_STRICT | ds.DS_PLAN_CHECK_MEMORY)
    plan_ms = (time.perf_counter() - t0) * 1e3
    info = ds.ds_plan_info(plan)
    payload = info["payload_bytes"]
    stream = torch.cuda.current_stream().cuda_stream
    ds.ds_config_set("variant", args.variant)

    # what this run's input was, so that it can be rebuilt: generator, seed, and the shard table as realised
    manifest_path = args.manifest or os.path.join(ROOT, "bench_out", f"manifest_{args.workload}.json")
    if manifest_path != "-":
        try:
            os.makedirs(os.path.dirname(os.path.abspath(manifest_path)), exist_ok=True)
            with open(manifest_path, "w") as f:
                json.dump({"workload": args.workload, "generator": f"workloads.by_name({args.workload!r})",
                           "name": w.name, "seed": w.seed, "align": w.align, "shards": n, "payload_bytes": payload,
                           "image_bytes": total, "arena_bytes": int(w.arena.size), "notes": w.notes,
                           "table": [{"name": sh.name, "dtype": sh.dtype, "shape": list(sh.shape),
                                      "strides": list(sh.strides), "byte_offset": sh.byte_offset,
                                      "tensor_id": sh.tensor_id, "file_offset": int(descs[i].file_offset),
                                      "nbytes": sh.nbytes} for i, sh in enumerate(w.shards)]}, f)
        except OSError as e:
            log(f"[bench] manifest not written: {e}")
            manifest_path = "-"

    if args.kernels_only:
        image_dev = torch.empty(max(total, 16), dtype=torch.uint8, device=dev)
        copy_src = torch.empty_like(image_dev)
        for _ in range(5):
            ds.ds_pack(plan, image_dev.data_ptr(), 0, total, stream)
        for _ in range(5):
            ds.ds_copy_probe(image_dev.data_ptr(), copy_src.data_ptr(), total & ~15, stream)
        for _ in range(5):
            ds.ds_unpack(plan, image_dev.data_ptr(), 0, total, stream)
        torch.cuda.synchronize()
        ds.ds_plan_destroy(plan)
        print(json.dumps({"kernels_only": True, "workload": args.workload, "image_bytes": total,
                          "payload_bytes": payload, "copy_probe_bytes": total & ~15}), flush=True)
        return 0

    # ---- measured link peak: best of 10 x 1 GiB contiguous device -> pinned host -------------
    probe_dev = torch.empty(GiB, dtype=torch.uint8, device=dev).random_(0, 255)
    probe_host = torch.empty(GiB, dtype=torch.uint8, pin_memory=True)
    link_best = 0.0
    for i in range(12):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        probe_host.copy_(probe_dev, non_blocking=True)
        b.record()
        torch.cuda.synchronize()
        if i >= 2:
            link_best = max(link_best, GiB / (a.elapsed_time(b) * 1e-3) / 1e9)
    h2d_best = 0.0
    for i in range(8):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        probe_dev.copy_(probe_host, non_blocking=True)
        b.record()
        torch.cuda.synchronize()
        if i >= 2:
            h2d_best = max(h2d_best, GiB / (a.elapsed_time(b) * 1e-3) / 1e9)
    del probe_dev, probe_host
    log(f"[bench] measured link peak: D2H {link_best:.1f} GB/s, H2D {h2d_best:.1f} GB/s")

    # ---- the timed region: K snapshots, back to back, each gated ------------------------------
    eng = ds.ds_engine_create(args.ring_bytes, args.chunk_bytes, args.stage_slot_bytes, args.stage_slots, 0,
                              ds.DS_ENGINE_AUTO_RELEASE, args.copy_streams, args.first_launch_bytes)

    def run_steps(k, pipelined=False):
        evs = []
        for _ in range(k):
            ev = ds.ds_snapshot_async(eng, plan, stream)
            ds.ds_event_wait_on_stream(ev, stream)       # gate before the (empty) update phase
            if not pipelined:
                ds.ds_event_wait(ev)                     # the whole image is in the host ring
            evs.append(ev)
        for ev in evs:
            ds.ds_event_wait(ev)
        return evs

    for ev in run_steps(args.warmup):
        ds.ds_event_destroy(ev)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    evs = run_steps(args.steps)
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
    ms_per_step = elapsed * 1e3 / args.steps
    value = payload * args.steps / elapsed / 1e9

    # algorithmic bytes of one gather launch: every payload byte read once, every image byte
    # (payload + padding) written once
    algo_bytes = payload + total
    achieved = algo_bytes * args.steps / (pack_ms * 1e-3) / 1e9 if pack_ms > 0 else 0.0
    # HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by what the same
    # counters read for ds_copy_probe): taken from the committed summary of that run, if there is one
    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"pmc_traffic_{args.workload}.md")
    if os.path.exists(tpath):
        import re
        m = re.search(r"traffic_bytes_per_launch\s*=\s*(\d+)", open(tpath).read())
        traffic = int(m.group(1)) if m else None
    roofline = {
        "bound": "hbm", "kernel": "ds_move_kernel<pack>",
        "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
        "launches": launches, "avg_launch_ms": round(pack_ms / max(launches, 1), 4),
        "algorithmic_bytes_per_launch": algo_bytes * args.steps // max(launches, 1),
    }
    if args.timed_only:
        ds.ds_engine_destroy(eng)
        ds.ds_plan_destroy(plan)
        print(json.dumps({"metric": "snapshot GB/s/GPU (pack+D2H to pinned host)", "value": round(value, 3),
                          "unit": "GB/s", "steps": args.steps, "warmup": args.warmup,
                          "ms_per_step": round(ms_per_step, 3), "workload": args.workload, "timed_only": True,
                          "roofline": roofline}), flush=True)
        return 0

    # one isolated snapshot: request -> whole image resident in the host ring
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev = ds.ds_snapshot_async(eng, plan, stream)
    ds.ds_event_wait(ev)
    latency_ms = (time.perf_counter() - t0) * 1e3
    one = ds.ds_event_stats(ev)
    ds.ds_event_destroy(ev)

    # the same steps without the per-step wait
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    pevs = run_steps(args.steps, pipelined=True)
    torch.cuda.synchronize()
    pipelined_gbps = payload * args.steps / (time.perf_counter() - t0) / 1e9
    for ev in pevs:
        ds.ds_event_destroy(ev)

    # ---- optional: the timeline of one snapshot, tier by tier ----------------------------------
    if args.timeline:
        eng_t = ds.ds_engine_create(args.ring_bytes, args.chunk_bytes, args.stage_slot_bytes, args.stage_slots, 0,
                                    ds.DS_ENGINE_AUTO_RELEASE | ds.DS_ENGINE_TRACE, args.copy_streams,
                                    args.first_launch_bytes)
        for _ in range(2):                                   # the second one is reported
            ev = ds.ds_snapshot_async(eng_t, plan, stream)
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
        lines = [f"# Timeline of one snapshot, workload {args.workload} (device clock, ms since the request)", "",
                 "Command:", "",
                 "    python3 bench.py " + " ".join(a for a in sys.argv[1:]), "",
                 f"image {total} B; ring slot / copy {args.chunk_bytes} B; staging {args.stage_slots} x "
                 f"{args.stage_slot_bytes} B; copy streams {args.copy_streams}", "",
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
                      f"the image is in the host ring at {tst['total_ms']:.3f} ms = {payload / tst['total_ms'] / 1e6:.2f} GB/s."]
        with open(args.timeline, "w") as f:
            f.write("\n".join(lines) + "\n")
        log(f"[bench] timeline written to {args.timeline}")

    # ---- gather and scatter alone, whole image, device to device ------------------------------
    image_dev = torch.empty(max(total, 16), dtype=torch.uint8, device=dev)

    def timed(fn, reps=20, warm=3):
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

    pack_med, pack_best = timed(lambda: ds.ds_pack(plan, image_dev.data_ptr(), 0, total, stream))
    unpack_med, unpack_best = timed(lambda: ds.ds_unpack(plan, image_dev.data_ptr(), 0, total, stream))
    copy_src = torch.empty_like(image_dev)
    nprobe = total & ~15
    probe_med, probe_best = timed(lambda: ds.ds_copy_probe(image_dev.data_ptr(), copy_src.data_ptr(), nprobe, stream))
    dtod_med, _ = timed(lambda: copy_src.copy_(image_dev))      # the runtime's own device-to-device copy
    del copy_src

    # ---- parity of this very run against the CPU oracle + the CPU baseline --------------------
    parity = "not checked"
    cpu_baseline = None
    if not args.no_cpu_baseline:
        from oracle import ds_oracle as orc
        tab = orc.table(w.shards, w.arena.ctypes.data)
        assert orc.layout(tab, n, w.align) == total
        want = np.empty(total, dtype=np.uint8)
        orc.pack(tab, n, total, threads=cores, out=want)          # also faults the pages in
        runs = []
        for _ in range(3):
            t0 = time.perf_counter()
            orc.pack(tab, n, total, threads=cores, out=want)
            runs.append(time.perf_counter() - t0)
        t0 = time.perf_counter()
        orc.pack(tab, n, total, threads=1, out=want)
        single = time.perf_counter() - t0
        cpu_baseline = {
            "value": round(payload / sorted(runs)[1] / 1e9, 2), "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": f"dso_pack_mt of the whole {args.workload} image ({payload / 1e9:.2f} GB), median of 3 runs "
                      f"after 1 warm-up, {cores} threads; single thread: {payload / single / 1e9:.2f} GB/s",
        }
        ds.ds_pack(plan, image_dev.data_ptr(), 0, total, stream)
        torch.cuda.synchronize()
        got = image_dev[:total].cpu().numpy()
        same = all(np.array_equal(got[lo:lo + (1 << 28)], want[lo:lo + (1 << 28)]) for lo in range(0, total, 1 << 28))
        parity = "byte-exact vs CPU oracle" if same else "MISMATCH vs CPU oracle"
        # restore: scatter the oracle's image back into a wiped arena, compare the whole arena
        keep = arena.clone()
        arena.fill_(0xA5)
        image_dev[:total].copy_(torch.from_numpy(want))
        ds.ds_unpack(plan, image_dev.data_ptr(), 0, total, stream)
        torch.cuda.synchronize()
        back = arena.cpu().numpy()
        w.arena[:] = 0xA5
        orc.unpack(tab, n, want)
        same_r = all(np.array_equal(back[lo:lo + (1 << 28)], w.arena[lo:lo + (1 << 28)])
                     for lo in range(0, back.size, 1 << 28))
        parity += "; restore byte-exact" if same_r else "; restore MISMATCH"
        # the same restore through the pipeline: host image -> ring slots -> staging -> scatter
        arena.fill_(0xA5)
        rev = ds.ds_restore_begin(eng, plan, stream)
        while True:
            slot = ds.ds_restore_next_slot(rev)
            if slot is None:
                break
            ptr, off, ln = slot
            ctypes.memmove(ptr, want[off:off + ln].ctypes.data, ln)
            ds.ds_restore_submit(rev, ptr)
        ds.ds_event_wait(rev)
        ds.ds_event_destroy(rev)
        back = arena.cpu().numpy()
        same_p = all(np.array_equal(back[lo:lo + (1 << 28)], w.arena[lo:lo + (1 << 28)])
                     for lo in range(0, back.size, 1 << 28))
        parity += "; pipelined restore byte-exact" if same_p else "; pipelined restore MISMATCH"
        arena.copy_(keep)
        del keep, got, back, want

    # restore pipeline rate with a null producer (slots submitted as they are: the link and the scatter)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    rev = ds.ds_restore_begin(eng, plan, stream)
    while True:
        slot = ds.ds_restore_next_slot(rev)
        if slot is None:
            break
        ds.ds_restore_submit(rev, slot[0])
    ds.ds_event_wait(rev)
    restore_s = time.perf_counter() - t0
    rst = ds.ds_event_stats(rev)
    ds.ds_event_destroy(rev)

    experiments = {}
    # ---- configs[4]: snapshots under a concurrent bf16 GEMM stream -----------------------------
    overlap = None
    if not args.no_overlap:
        M = 8192
        A = torch.randn(M, M, device=dev, dtype=torch.bfloat16)
        B = torch.randn(M, M, device=dev, dtype=torch.bfloat16)
        C = torch.empty(M, M, device=dev, dtype=torch.bfloat16)
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
        G = max(4, int(round(1.5 * one["total_ms"] / gemm_ms)))   # forward/backward ~1.5x one snapshot

        def loop(with_snapshots: bool, G: int = G, eng=eng):
            evs = []
            prev = None
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            loop.gate_host_ms = 0.0
            torch.cuda.synchronize()
            w0 = time.perf_counter()
            a.record()
            for _ in range(args.gemm_iters):
                for _ in range(G):                                # state is only read here
                    torch.matmul(A, B, out=C)
                if prev is not None:
                    g0 = time.perf_counter()
                    ds.ds_event_wait_on_stream(prev, stream)      # the lazy gate
                    loop.gate_host_ms += (time.perf_counter() - g0) * 1e3
                arena.add_(1)                                     # the mutating update phase
                if with_snapshots:
                    prev = ds.ds_snapshot_async(eng, plan, stream)
                    evs.append(prev)
            b.record()
            torch.cuda.synchronize()
            for ev in evs:
                ds.ds_event_wait(ev)
                ds.ds_event_destroy(ev)
            loop.wall_ms = (time.perf_counter() - w0) * 1e3      # until the last snapshot is in the host ring
            return a.elapsed_time(b)

        loop(True)
        base = min(loop(False) for _ in range(2))
        with_s = min(loop(True) for _ in range(2))
        blocked_ms = max(with_s - base, 1e-6) / args.gemm_iters
        overlap = {
            # the paper's measure (Sec. VI-D, scaling of model sizes): checkpoint size over the time training is blocked by it
            "blocked_ms_per_iter": round(blocked_ms, 4),
            "effective_checkpoint_GBps": round(payload / blocked_ms / 1e6, 1),
            "gate_call_host_ms_per_iter": round(loop.gate_host_ms / args.gemm_iters, 4),
            "gemm": "bf16 8192x8192x8192 (torch.matmul)", "gemm_ms": round(gemm_ms, 3),
            "gemm_tflops": round(2 * M ** 3 / gemm_ms / 1e9, 1), "gemms_per_iter": G, "iters": args.gemm_iters,
            "ms_without_snapshots": round(base, 2), "ms_with_snapshots": round(with_s, 2),
            "slowdown_pct": round(100.0 * (with_s - base) / base, 2),
            "ring_bytes": args.ring_bytes,
        }
        # stress point: a compute window far shorter than one snapshot, so every gate stalls and the
        # loop runs at the pace of the link (back-pressure of the ring and the staging slots)
        Gs = max(1, G // 6)
        base_s = min(loop(False, Gs) for _ in range(2))
        with_ss = loop(True, Gs)
        overlap["stress"] = {
            "gemms_per_iter": Gs, "ms_without_snapshots": round(base_s, 2), "ms_with_snapshots": round(with_ss, 2),
            "wall_ms_until_last_snapshot_done": round(loop.wall_ms, 2),
            "snapshot_GBps_sustained": round(payload * args.gemm_iters / loop.wall_ms / 1e6, 2),
            "note": "compute window 1/6 of the default: the gate and the staging slots make the loop wait for the link",
        }
        if args.experiments:
            # capture variants, measured only.  (1) The gather limited to a few resident work-groups: does a
            # slower, narrower gather disturb the GEMM stream less?
            experiments["grid_limited_gather"] = []
            for limit in (4096, 1024, 256):
                eng_x = ds.ds_engine_create(args.ring_bytes, args.chunk_bytes, args.stage_slot_bytes, args.stage_slots,
                                            limit, ds.DS_ENGINE_AUTO_RELEASE, args.copy_streams, args.first_launch_bytes)
                ev = ds.ds_snapshot_async(eng_x, plan, stream)
                ds.ds_event_wait(ev)
                st = ds.ds_event_stats(ev)
                ds.ds_event_destroy(ev)
                loop(True, G, eng_x)
                with_x = min(loop(True, G, eng_x) for _ in range(2))
                experiments["grid_limited_gather"].append({
                    "resident_workgroups": limit, "gather_ms": round(st["pack_ms"], 3),
                    "capture_ms": round(st["capture_ms"], 3),
                    "slowdown_pct": round(100.0 * (with_x - base) / base, 2)})
                ds.ds_engine_destroy(eng_x)
        del A, B, C

    if args.experiments:
        # (2) No staging and no copy: the gather writes straight into pinned host memory over the link.
        host_img = torch.empty(max(total, 16), dtype=torch.uint8, pin_memory=True)
        d_med, d_best = timed(lambda: ds.ds_pack(plan, host_img.data_ptr(), 0, total, stream), reps=5, warm=1)
        ok = None
        if not args.no_cpu_baseline:
            from oracle import ds_oracle as orc
            arena.copy_(torch.from_numpy(w.arena))        # the overlap leg has mutated the tensors: same bytes on both sides
            ds.ds_pack(plan, host_img.data_ptr(), 0, total, stream)
            torch.cuda.synchronize()
            tab = orc.table(w.shards, w.arena.ctypes.data)
            assert orc.layout(tab, n, w.align) == total
            want = orc.pack(tab, n, total, threads=cores)
            got = host_img[:total].numpy()
            ok = all(np.array_equal(got[lo:lo + (1 << 28)], want[lo:lo + (1 << 28)]) for lo in range(0, total, 1 << 28))
            del want
        direct = {
            "ms": round(d_med, 3), "GBps": round(payload / d_med / 1e6, 2), "best_GBps": round(payload / d_best / 1e6, 2),
            "byte_exact_vs_oracle": ok,
            "note": "the kernel holds the tensors for the whole transfer, so the gate opens after this time, "
                    "not after the 0.5 ms of the staged gather; resident_workgroups 0 = one work-group per chunk"}
        if overlap is not None:
            side = torch.cuda.Stream()                    # default priority

            def loop_direct():
                prev = None
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                a.record()
                for _ in range(args.gemm_iters):
                    for _ in range(overlap["gemms_per_iter"]):
                        torch.matmul(gA, gB, out=gC)
                    if prev is not None:
                        torch.cuda.current_stream().wait_event(prev)   # the gate: the whole transfer
                    arena.add_(1)
                    req = torch.cuda.Event()
                    req.record()
                    side.wait_event(req)
                    ds.ds_pack(plan, host_img.data_ptr(), 0, total, side.cuda_stream)
                    prev = torch.cuda.Event()
                    prev.record(side)
                b.record()
                torch.cuda.synchronize()
                return a.elapsed_time(b)

            M = 8192
            gA = torch.randn(M, M, device=dev, dtype=torch.bfloat16)
            gB = torch.randn(M, M, device=dev, dtype=torch.bfloat16)
            gC = torch.empty(M, M, device=dev, dtype=torch.bfloat16)
            direct["under_gemms"] = []
            for limit in (0, 1024, 256, 64, 16):
                ds.ds_config_set("grid_limit", limit)
                x_med, _ = timed(lambda: ds.ds_pack(plan, host_img.data_ptr(), 0, total, stream), reps=3, warm=1)
                loop_direct()
                with_d = min(loop_direct() for _ in range(2))
                direct["under_gemms"].append({
                    "resident_workgroups": limit, "alone_GBps": round(payload / x_med / 1e6, 2),
                    "gemm_slowdown_pct": round(100.0 * (with_d - overlap["ms_without_snapshots"]) /
                                               overlap["ms_without_snapshots"], 2)})
            ds.ds_config_set("grid_limit", 0)
            del gA, gB, gC
        experiments["gather_into_pinned_host"] = direct
        del host_img

    if args.experiments:
        # (3) Differential snapshot (the paper's future work): keep the previous image in HBM, gather the new
        # one beside it, compare them chunk by chunk on the device, copy only the chunks that changed.
        cb = args.chunk_bytes
        n_blocks = -(-total // cb)
        img_a = torch.empty(max(total, 16), dtype=torch.uint8, device=dev)
        img_b = torch.empty(max(total, 16), dtype=torch.uint8, device=dev)
        flags_dev = torch.zeros(n_blocks, dtype=torch.int32, device=dev)
        host_img = torch.empty(max(total, 16), dtype=torch.uint8, pin_memory=True)
        keep = arena.clone()
        rows = []
        for frac in (1.0, 0.25, 0.05, 0.0):
            # the reference: image of the unchanged state, on the device and (whole) in host memory
            arena.copy_(keep)
            ds.ds_pack(plan, img_a.data_ptr(), 0, total, stream)
            torch.cuda.synchronize()
            host_img[:total].copy_(img_a[:total])
            n_mut = int(arena.numel() * frac)
            if n_mut:
                arena[:n_mut].add_(1)                                  # this share of the rank's memory changes
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ds.ds_pack(plan, img_b.data_ptr(), 0, total, stream)
            ds.ds_image_diff(img_a.data_ptr(), img_b.data_ptr(), total, cb, flags_dev.data_ptr(), stream)
            dirty = flags_dev.cpu().nonzero().flatten().tolist()       # the one host synchronisation
            for k in dirty:
                lo, hi = k * cb, min((k + 1) * cb, total)
                host_img[lo:hi].copy_(img_b[lo:hi], non_blocking=True)
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3
            ok = bool(torch.equal(host_img[:total], img_b[:total].cpu()))   # the host image is the new image
            rows.append({"share_of_memory_changed": frac, "dirty_chunks": len(dirty), "chunks": n_blocks,
                         "ms": round(ms, 3), "effective_GBps": round(payload / ms / 1e6, 1),
                         "host_image_equals_new_image": ok})
        arena.copy_(keep)
        experiments["differential_snapshot"] = {
            "rows": rows,
            "note": "gather + device compare of two images (ds_image_diff, one flag per ring-slot-sized chunk) + "
                    "copies of the changed chunks only; costs a second image in HBM and one host synchronisation"}
        del img_a, img_b, host_img, keep

    file_plans = []
    if args.experiments:
        # (4) One rank's checkpoint split over several files (the paper's 7B rank writes 20, Sec. VI-D): one plan
        # per file over consecutive shards of about equal bytes, all through the one engine, back to back.
        F = min(args.files, n)
        cuts, acc, sizes = [0], 0, [ds.ds_plan_shard(plan, i)[3] for i in range(n)]
        for i in range(n):
            acc += sizes[i]
            if acc >= payload * len(cuts) / F and len(cuts) < F and i + 1 < n:
                cuts.append(i + 1)
        cuts.append(n)
        for a, b in zip(cuts[:-1], cuts[1:]):
            dg = ds.make_descs(w.shards[a:b], arena.data_ptr())
            ds.ds_layout_assign(dg, b - a, w.align)
            file_plans.append(ds.ds_plan_create(dg, b - a, w.align, ds.DS_PLAN_STRICT))

        def several():
            t0 = time.perf_counter()
            evs = [ds.ds_snapshot_async(eng, pl, stream) for pl in file_plans]
            ds.ds_event_wait_on_stream(evs[-1], stream)      # snapshots run in order: the last gate covers all
            ds.ds_event_wait_captured(evs[-1])
            t_cap = time.perf_counter() - t0                 # first request -> every tensor may be mutated (host clock)
            for ev in evs:
                ds.ds_event_wait(ev)
            return evs, t_cap, time.perf_counter() - t0
        for ev in several()[0]:
            ds.ds_event_destroy(ev)
        torch.cuda.synchronize()
        evs, cap_s, several_s = several()
        cap = cap_s * 1e3
        for ev in evs:
            ds.ds_event_destroy(ev)
        experiments["rank_state_as_several_plans"] = {
            "plans": len(file_plans), "smallest_image_bytes": min(ds.ds_plan_info(pl)["total_bytes"] for pl in file_plans),
            "largest_image_bytes": max(ds.ds_plan_info(pl)["total_bytes"] for pl in file_plans),
            "GBps_into_host_ring": round(payload / several_s / 1e9, 2),
            "first_request_to_all_captured_ms": round(cap, 3),
            "note": "the same bytes as one image, requested as one snapshot per file; compare with `value`"}

    ds.ds_engine_destroy(eng)
    torch.cuda.synchronize()

    # ---- the checkpoint file: snapshot -> ring -> tensor region (writer threads) with an object log
    # appended behind it at the same time, trailer last; then file -> ring -> GPU ---------------
    file_tier = None
    if not args.no_file:
        import threading
        eng2 = ds.ds_engine_create(args.ring_bytes, args.chunk_bytes, args.stage_slot_bytes, args.stage_slots, 0, 0,
                                   args.copy_streams, args.first_launch_bytes)
        obj_chunk = os.urandom(64 << 10)
        n_obj_threads, chunks_per_thread = 2, 128             # 16 MiB of serialized objects in 64 KiB chunks

        def one_dir(d):
            path = os.path.join(d, f"ds_bench_{os.getpid()}.ckpt")
            try:
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                ev = ds.ds_snapshot_async(eng2, plan, stream)
                ck = ds.ds_ckpt_create(path, plan, ds.DS_FILE_DIRECT |
                                       (ds.DS_FILE_URING if args.file_engine == "uring" else 0))
                ds.ds_ckpt_flush_snapshot(ck, ev, args.file_threads)

                def objects(t):
                    for k in range(chunks_per_thread):
                        ds.ds_ckpt_append(ck, 1000 + t * 16 + k % 16, obj_chunk)
                ts = [threading.Thread(target=objects, args=(t,)) for t in range(n_obj_threads)]
                for t in ts:
                    t.start()
                ds.ds_event_wait_on_stream(ev, stream)
                for t in ts:
                    t.join()
                nbytes, _ = ds.ds_ckpt_finish(ck)
                flush_s = time.perf_counter() - t0
                ds.ds_event_wait(ev)
                fst = ds.ds_event_stats(ev)
                ds.ds_event_destroy(ev)
                t0 = time.perf_counter()
                rd = ds.ds_ckpt_open(path)
                rev = ds.ds_ckpt_restore(rd, eng2, plan, args.file_threads, ds.DS_FILE_DIRECT, stream)
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
            file_tier = {"threads": args.file_threads, "engine": args.file_engine,
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
                        ev = ds.ds_snapshot_async(eng2, pl, stream)
                        ck = ds.ds_ckpt_create(path, pl, ds.DS_FILE_DIRECT |
                                               (ds.DS_FILE_URING if args.file_engine == "uring" else 0))
                        ds.ds_ckpt_flush_snapshot(ck, ev, max(1, args.file_threads // 2))
                        evs.append(ev)
                        cks.append(ck)
                    ds.ds_event_wait_on_stream(evs[-1], stream)
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
    torch.cuda.synchronize()
    for pl in file_plans:
        ds.ds_plan_destroy(pl)
    ds.ds_plan_destroy(plan)

    out = {
        "metric": "snapshot GB/s/GPU (pack+D2H to pinned host)",
        "value": round(value, 3), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {
            "workload": f"{args.workload}: {WORKLOADS[args.workload]}", "payload_bytes": payload,
            "image_bytes": total, "shards": n, "align": w.align, "host_ring_bytes": args.ring_bytes,
            "d2h_chunk_bytes": args.chunk_bytes, "stage_slot_bytes": args.stage_slot_bytes,
            "stage_slots": args.stage_slots, "copy_streams": args.copy_streams,
            "first_launch_bytes": args.first_launch_bytes,
            "workgroup_chunk_bytes": info["chunk_bytes"],
            "manifest": None if manifest_path == "-" else os.path.relpath(manifest_path, ROOT),
        },
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "parity": parity,
        "d2h": {"achieved_GBps": round(total * args.steps / (copy_ms * 1e-3) / 1e9, 2),
                "link_peak_measured_GBps": round(link_best, 2),
                "frac": round(total * args.steps / (copy_ms * 1e-3) / 1e9 / link_best, 4)},
        "snapshot_latency_ms": round(latency_ms, 3),
        "pipelined_GBps": round(pipelined_gbps, 3),
        "capture_ms": round(capture_ms / args.steps, 3),          # request -> tensors may be mutated
        "submit_host_ms": round(submit_ms / args.steps, 4),       # host time inside ds_snapshot_async
        "plan_create_ms": round(plan_ms, 3),
        "standalone": {
            "pack_ms": round(pack_med, 4), "pack_GBps": round(algo_bytes / pack_med / 1e6, 1),
            "pack_best_GBps": round(algo_bytes / pack_best / 1e6, 1),
            "unpack_ms": round(unpack_med, 4), "unpack_GBps": round(2 * payload / unpack_med / 1e6, 1),
            "copy_probe_GBps": round(2 * nprobe / probe_med / 1e6, 1),    # plain copy, same shape: the ceiling
            "runtime_d2d_copy_GBps": round(2 * total / dtod_med / 1e6, 1),   # torch copy_ (hipMemcpy device to device)
            "pack_vs_copy_probe": round((algo_bytes / pack_med) / (2 * nprobe / probe_med), 4),
        },
        "restore": {"GBps_null_producer": round(payload / restore_s / 1e9, 2), "ms": round(restore_s * 1e3, 3),
                    "h2d_link_peak_measured_GBps": round(h2d_best, 2),
                    "frac_of_h2d_peak": round(payload / restore_s / 1e9 / h2d_best, 4),
                    "scatter_ms": round(rst["pack_ms"], 3), "scatter_launches": rst["n_pack_launches"]},
        "overlap": overlap,
        "file_tier": file_tier,
        **({"experiments": experiments} if experiments else {}),
        "device": {"name": props.name, "compute_units": props.multi_processor_count,
                   "hbm_bytes": props.total_memory},
        "hip_runtime": ds.hip_runtime_in_use(),
    }
    print(json.dumps(out), flush=True)
    return 0 if "MISMATCH" not in parity else 1


if __name__ == "__main__":
    sys.exit(main())
