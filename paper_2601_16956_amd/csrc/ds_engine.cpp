// The snapshot engine: lazy, non-blocking capture of one GPU's shards into a
// pre-pinned host ring (DataStates-LLM Sec. V-A1, V-A2, V-A4; implementation
// notes of Sec. V-C: pinned circular buffer, dedicated streams, background
// host thread).
//
// Data path of one snapshot, image bytes [0, T):
//
//   compute stream --E_requested--> gather stream: one gather launch per
//   stage_slot_bytes of image (optionally a shorter first launch, so that the
//   link starts working sooner)  --E_packed--> copy stream(s): one hipMemcpyAsync
//   per ring slot, device staging -> pinned ring  --E_done[slot]--> consumer.
//
// Device staging is one ring of bytes: a gather launch takes the next piece of it,
// after the copies that last read those bytes.  Gathers are issued ahead of the
// copies as far as staging has room -- across queued snapshots too -- so when
// staging holds what has been requested (a rank's whole state, written as several
// files = several snapshots, say) every gate opens after the gathers alone, however
// far behind the link, the host ring or the storage are.
//
// The caller's stream is touched twice only: the record at the request and the
// wait at the gate.  The gate waits for the LAST GATHER, not for the last
// copy: once every source byte sits in staging the tensors may be mutated.
// MI355X has HBM to spare (288 GB), so staging as large as the image is an
// ordinary setting and the update phase is then delayed by the gather time
// only (a fraction of a millisecond per GB), not by the link.
#include <algorithm>
#include <chrono>
#include <condition_variable>
#include <deque>
#include <list>
#include <mutex>
#include <new>
#include <thread>

#include "ds_internal.h"

namespace {
constexpr int kMaxCopyStreams = 2;

// The pinned ring of a destroyed engine is kept for the next engine of the process (one allocation, the
// largest seen): pinning 2 GiB takes hundreds of milliseconds, and -- measured -- a ring allocated later in a
// process's life, when the first one has been freed, can be backed by memory the link writes at 30 GB/s
// instead of 57 (its later slots; the first allocation of a process does not show it).  The paper's pool is
// allocated and pinned once and reused by every request (Sec. V-A1); this extends that to engines.
struct PinnedCache {
  std::mutex mu;
  uint8_t *ptr = nullptr;
  uint64_t bytes = 0;
} g_pinned;

hipError_t ring_alloc(uint64_t need, uint8_t **out, uint64_t *cap) {
  {
    std::lock_guard<std::mutex> lk(g_pinned.mu);
    if (g_pinned.ptr && g_pinned.bytes >= need) {
      *out = g_pinned.ptr;
      *cap = g_pinned.bytes;
      g_pinned.ptr = nullptr;
      g_pinned.bytes = 0;
      return hipSuccess;
    }
  }
  *cap = need;
  return hipHostMalloc((void **)out, need, hipHostMallocPortable);
}

// The same for the device staging: device memory that has just been allocated is slow on first touch (the
// first snapshot or restore of a new engine ran at 30-50 GB/s instead of 56), so an engine hands its staging
// on to the next one of the process on the same device.
struct StageCache {
  std::mutex mu;
  uint8_t *ptr = nullptr;
  uint64_t bytes = 0;
  int device = -1;
} g_stage;

hipError_t stage_alloc(int dev, uint64_t need, uint8_t **out, uint64_t *cap) {
  {
    std::lock_guard<std::mutex> lk(g_stage.mu);
    if (g_stage.ptr && g_stage.device == dev && g_stage.bytes >= need) {
      *out = g_stage.ptr;
      *cap = g_stage.bytes;
      g_stage.ptr = nullptr;
      g_stage.bytes = 0;
      return hipSuccess;
    }
  }
  *cap = need;
  return hipMalloc((void **)out, need);
}

void stage_free(int dev, uint8_t *p, uint64_t cap) {
  {
    std::lock_guard<std::mutex> lk(g_stage.mu);
    if (!g_stage.ptr || (g_stage.device == dev && cap > g_stage.bytes)) {
      std::swap(p, g_stage.ptr);
      std::swap(cap, g_stage.bytes);
      g_stage.device = dev;
    }
  }
  if (p) (void)hipFree(p);
}

void ring_free(uint8_t *p, uint64_t cap) {
  {
    std::lock_guard<std::mutex> lk(g_pinned.mu);
    if (!g_pinned.ptr || cap > g_pinned.bytes) {
      std::swap(p, g_pinned.ptr);
      std::swap(cap, g_pinned.bytes);
    }
  }
  if (p) (void)hipHostFree(p);
}

// The streams of a destroyed engine are kept for the next engine of the process on the same device.  The
// runtime spreads streams over a few hardware queues in the order they are created; measured, the two copy
// streams of an engine created later in a process's life (after other engines' streams had been created and
// destroyed) shared the link 2:1 instead of 1:1 and the snapshot ran at 45 GB/s instead of 56.  Reusing the
// first engine's streams keeps the mapping the first engine had.
struct PooledStream {
  int device;
  uint64_t id;  // order of creation: an engine takes the oldest idle ones, so the roles (gather, copy 0, copy 1)
                // fall to the same streams from one engine to the next
  hipStream_t stream;
};
struct StreamPool {
  std::mutex mu;
  std::vector<PooledStream> idle;
  uint64_t next_id = 0;
} g_streams;

hipError_t stream_take(int dev, PooledStream *out) {
  {
    std::lock_guard<std::mutex> lk(g_streams.mu);
    size_t best = g_streams.idle.size();
    for (size_t i = 0; i < g_streams.idle.size(); ++i)
      if (g_streams.idle[i].device == dev && (best == g_streams.idle.size() || g_streams.idle[i].id < g_streams.idle[best].id))
        best = i;
    if (best < g_streams.idle.size()) {
      *out = g_streams.idle[best];
      g_streams.idle.erase(g_streams.idle.begin() + (long)best);
      return hipSuccess;
    }
    out->id = g_streams.next_id++;
  }
  out->device = dev;
  return hipStreamCreateWithFlags(&out->stream, hipStreamNonBlocking);
}

void stream_give(const PooledStream &s) {
  if (!s.stream) return;
  try {
    std::lock_guard<std::mutex> lk(g_streams.mu);
    g_streams.idle.push_back(s);
  } catch (const std::bad_alloc &) {
    (void)hipStreamDestroy(s.stream);
  }
}
}  // namespace

// frees the cached ring and staging (ds_config_set("drop_pinned_cache", 1))
void ds_drop_pinned_cache() {
  uint8_t *p = nullptr, *d = nullptr;
  {
    std::lock_guard<std::mutex> lk(g_pinned.mu);
    std::swap(p, g_pinned.ptr);
    g_pinned.bytes = 0;
  }
  {
    std::lock_guard<std::mutex> lk(g_stage.mu);
    std::swap(d, g_stage.ptr);
    g_stage.bytes = 0;
  }
  if (p) (void)hipHostFree(p);
  if (d) (void)hipFree(d);
}

struct ds_event;

// A piece of staging that a gather launch has filled (or is about to).
struct StageRegion {
  uint64_t off = 0, len = 0;
  bool copies_enqueued = false;  // the copies that read it have been enqueued and `done` recorded behind them
  int n_done = 0;
  hipEvent_t done[kMaxCopyStreams] = {nullptr, nullptr};
};

struct ds_engine {
  int device = 0;
  uint32_t flags = 0;
  uint32_t grid_limit = 0;
  uint64_t chunk_bytes = 0;       // ring slot = one copy
  uint64_t stage_slot_bytes = 0;  // image bytes per gather launch
  uint64_t first_launch_bytes = 0; // image bytes of the first gather launch of a snapshot
  uint32_t stage_slots = 0;
  // a restore scatters staging in pieces of this many image bytes (a few copies' worth: the scatter of one
  // piece then runs beside the copies of the next, and only the last, short one is left over at the end)
  uint64_t restore_piece_bytes = 0;
  uint32_t restore_pieces = 0;    // pieces of that size that staging holds
  uint32_t ring_slots = 0;
  int n_copy_streams = 1;
  hipStream_t pack_stream = nullptr;
  hipStream_t copy_stream[kMaxCopyStreams] = {nullptr, nullptr};
  uint8_t *stage = nullptr;  // device
  uint8_t *ring = nullptr;   // pinned host
  uint64_t ring_cap = 0;     // bytes of the allocation behind `ring` (it may come from the process's cache)
  uint64_t stage_cap = 0;    // the same for `stage`
  // engine-owned events, reused by every snapshot
  std::vector<hipEvent_t> ring_done;                    // copy into ring slot r finished
  std::vector<uint8_t> ring_busy;  // consumer mode: slot holds data not yet released
  std::vector<int8_t> ring_stream; // copy stream that last wrote the slot (-1: none yet)
  uint32_t ring_next = 0;
  uint64_t copies_issued = 0;
  // staging as a ring of bytes (touched by the engine thread; by a restore only while the engine is idle)
  uint64_t stage_bytes = 0, stage_head = 0;
  std::list<StageRegion> regions;      // pieces of staging whose last gather may still be read by copies
  std::vector<hipEvent_t> event_pool;  // spare events of regions that have been taken over

  std::vector<PooledStream> pooled;  // the streams above, as taken from the process's pool

  std::mutex mu;
  std::condition_variable cv;
  std::deque<ds_event *> queue;
  bool stop = false;
  int live_events = 0;
  bool restoring = false;  // a restore event is alive: ring and staging are its own
  std::thread worker;
};

struct DsChunk {
  uint64_t file_off = 0, len = 0;
  uint32_t ring_slot = 0;
  int state = 0;  // 0 not issued, 1 copy issued, 2 handed to the consumer, 3 released
};

struct ds_event {
  ds_engine *eng = nullptr;
  const ds_plan *plan = nullptr;
  hipEvent_t requested = nullptr, captured = nullptr, final_ev = nullptr, copy_begin = nullptr;
  std::vector<hipEvent_t> pack_begin, pack_end;
  std::vector<uint64_t> pack_lo, pack_hi;          // image range of each gather launch
  std::vector<hipEvent_t> copy_b, copy_e;           // DS_ENGINE_TRACE: around every chunk's copy
  std::vector<DsChunk> chunks;
  uint32_t cursor = 0;  // next chunk the consumer gets
  bool capture_issued = false;  // the last gather (and the `captured` event) is enqueued
  bool all_issued = false;
  int error = DS_OK;
  double submit_host_ms = 0;
  // restore (host image -> tensors): chunks are handed to the producer, submitted, copied up, scattered
  bool restore = false;
  uint32_t r_handed = 0, r_submitted = 0;
  std::vector<hipEvent_t> group_done;  // scatter of staging group gi finished
};

const ds_plan *ds_event_plan(const ds_event *ev) { return ev ? ev->plan : nullptr; }

namespace {

int hip_fail(hipError_t e) {
  ds_set_hip_error(e);
  return DS_EHIP;
}

#define W_TRY(expr)                          \
  do {                                       \
    hipError_t _e = (expr);                  \
    if (_e != hipSuccess) return hip_fail(_e); \
  } while (0)

// One snapshot in the hands of the engine thread.
struct Job {
  ds_event *ev = nullptr;
  struct Group {
    uint64_t lo = 0, hi = 0;  // image range of one gather launch
    std::list<StageRegion>::iterator region;
  };
  std::vector<Group> groups;
  bool prepared = false;
  size_t np = 0;             // gathers issued
  size_t nc = 0;             // groups whose copies have all been issued
  bool group_begun = false;  // the copy streams already wait for the gather of group nc
  uint64_t at = 0;           // image offset of the next copy of group nc
  uint32_t k = 0;            // its chunk number
  int ncs = 1;               // copy streams this snapshot uses
};

int pool_event(ds_engine *g, hipEvent_t *out) {
  if (!g->event_pool.empty()) {
    *out = g->event_pool.back();
    g->event_pool.pop_back();
    return DS_OK;
  }
  W_TRY(hipEventCreateWithFlags(out, hipEventDisableTiming));
  return DS_OK;
}

void recycle_region(ds_engine *g, StageRegion &r) {
  for (int c = 0; c < kMaxCopyStreams; ++c)
    if (r.done[c]) {
      g->event_pool.push_back(r.done[c]);
      r.done[c] = nullptr;
    }
}

void forget_regions(ds_engine *g) {
  for (StageRegion &r : g->regions) recycle_region(g, r);
  g->regions.clear();
  g->stage_head = 0;
}

int mark_captured(ds_engine *g, ds_event *ev) {
  W_TRY(hipEventRecord(ev->captured, g->pack_stream));
  {
    std::lock_guard<std::mutex> lk(g->mu);
    ev->capture_issued = true;
  }
  g->cv.notify_all();
  return DS_OK;
}

int prepare_job(ds_engine *g, Job &j) {
  ds_event *ev = j.ev;
  const uint64_t T = ev->plan->total_bytes;
  j.prepared = true;
  W_TRY(hipEventCreate(&ev->captured));
  W_TRY(hipEventCreate(&ev->final_ev));
  W_TRY(hipEventCreate(&ev->copy_begin));
  for (uint64_t at = 0; at < T;) {
    // the first launch may be shorter than the others (first_launch_bytes)
    const uint64_t want = j.groups.empty() ? g->first_launch_bytes : g->stage_slot_bytes;
    Job::Group gr;
    gr.lo = at;
    gr.hi = at + want < T ? at + want : T;
    j.groups.push_back(gr);
    at = gr.hi;
  }
  // A snapshot of only a few chunks keeps to one copy stream: there is no gap between copies for the
  // second stream to hide, so the events that would tie it in are saved.
  j.ncs = ev->chunks.size() < 4 ? 1 : g->n_copy_streams;
  if (j.groups.empty()) {
    W_TRY(hipStreamWaitEvent(g->pack_stream, ev->requested, 0));
    return mark_captured(g, ev);
  }
  return DS_OK;
}

// The next gather of the snapshot, if staging has room for it: *issued = false means that the bytes it
// would take are still waiting for copies that have not been enqueued yet.
int try_issue_pack(ds_engine *g, Job &j, bool *issued) {
  ds_event *ev = j.ev;
  Job::Group &gr = j.groups[j.np];
  const uint64_t len = gr.hi - gr.lo;
  uint64_t off = g->stage_head;
  if (off + len > g->stage_bytes) off = 0;  // a launch's piece is contiguous: the rest of the ring's end stays unused
  auto overlaps = [&](const StageRegion &r) { return r.off < off + len && off < r.off + r.len; };
  for (const StageRegion &r : g->regions)
    if (overlaps(r) && !r.copies_enqueued) {
      *issued = false;
      return DS_OK;
    }
  if (j.np == 0) W_TRY(hipStreamWaitEvent(g->pack_stream, ev->requested, 0));
  for (auto it = g->regions.begin(); it != g->regions.end();) {
    if (overlaps(*it)) {
      for (int c = 0; c < it->n_done; ++c) W_TRY(hipStreamWaitEvent(g->pack_stream, it->done[c], 0));
      recycle_region(g, *it);
      it = g->regions.erase(it);
    } else {
      ++it;
    }
  }
  g->regions.emplace_back();
  gr.region = std::prev(g->regions.end());
  gr.region->off = off;
  gr.region->len = len;
  g->stage_head = off + len;
  hipEvent_t b, e;
  W_TRY(hipEventCreate(&b));
  ev->pack_begin.push_back(b);
  W_TRY(hipEventCreate(&e));
  ev->pack_end.push_back(e);
  ev->pack_lo.push_back(gr.lo);
  ev->pack_hi.push_back(gr.hi);
  W_TRY(hipEventRecord(b, g->pack_stream));
  int rc = ds_launch_move(ev->plan, true, g->stage + off, gr.lo, gr.hi, g->grid_limit, g->pack_stream);
  if (rc != DS_OK) return rc;
  W_TRY(hipEventRecord(e, g->pack_stream));
  *issued = true;
  if (++j.np == j.groups.size()) return mark_captured(g, ev);
  return DS_OK;
}

// Copies of the snapshot's next group whose gather has been issued.  Returns after one group, or earlier
// with *blocked = true when the host ring is full and a new request has arrived: its gathers need not wait
// for the ring.
int issue_group_copies(ds_engine *g, Job &j, bool *blocked) {
  ds_event *ev = j.ev;
  if (j.nc >= j.np) return DS_OK;
  Job::Group &gr = j.groups[j.nc];
  uint8_t *slot = g->stage + gr.region->off;
  const int ncs = j.ncs;
  if (!j.group_begun) {
    for (int c = 0; c < ncs; ++c) W_TRY(hipStreamWaitEvent(g->copy_stream[c], ev->pack_end[j.nc], 0));
    if (j.nc == 0) W_TRY(hipEventRecord(ev->copy_begin, g->copy_stream[0]));
    j.at = gr.lo;
    j.group_begun = true;
  }
  for (; j.at < gr.hi; j.at += g->chunk_bytes, ++j.k) {
    const uint64_t lo = j.at;
    const uint64_t len = lo + g->chunk_bytes < gr.hi ? g->chunk_bytes : gr.hi - lo;
    uint32_t r;
    {
      std::unique_lock<std::mutex> lk(g->mu);
      r = g->ring_next;
      if (!(g->flags & DS_ENGINE_AUTO_RELEASE)) {
        // back-pressure: the ring is full until the consumer releases a slot
        g->cv.wait(lk, [&] { return !g->ring_busy[r] || !g->queue.empty(); });
        if (g->ring_busy[r]) {
          *blocked = true;
          return DS_OK;
        }
        g->ring_busy[r] = 1;
      }
      g->ring_next = (r + 1) % g->ring_slots;
    }
    const int c = (int)(g->copies_issued++ % (uint64_t)ncs);
    hipStream_t cs = g->copy_stream[c];
    // The slot's previous copy must have run.  On the same stream it has (a stream runs its copies in
    // order); only a copy that ran on the other stream needs a wait.  (A wait for an event that has not fired
    // yet puts a barrier into the stream; with a ring shorter than the image every copy would carry one, and
    // the copies then run at 85 % of the link instead of 99 %.)
    if (g->ring_stream[r] >= 0 && g->ring_stream[r] != c) W_TRY(hipStreamWaitEvent(cs, g->ring_done[r], 0));
    g->ring_stream[r] = (int8_t)c;
    if (g->flags & DS_ENGINE_TRACE) {
      hipEvent_t tb, te;
      W_TRY(hipEventCreate(&tb));
      ev->copy_b.push_back(tb);
      W_TRY(hipEventCreate(&te));
      ev->copy_e.push_back(te);
      W_TRY(hipEventRecord(tb, cs));
    }
    W_TRY(hipMemcpyAsync(g->ring + (uint64_t)r * g->chunk_bytes, slot + (lo - gr.lo), len, hipMemcpyDeviceToHost, cs));
    if (g->flags & DS_ENGINE_TRACE) W_TRY(hipEventRecord(ev->copy_e.back(), cs));
    W_TRY(hipEventRecord(g->ring_done[r], cs));
    {
      std::lock_guard<std::mutex> lk(g->mu);
      ev->chunks[j.k].ring_slot = r;
      ev->chunks[j.k].state = 1;
    }
    g->cv.notify_all();
  }
  // the piece of staging may be gathered into again once these copies have run
  for (int c = 0; c < ncs; ++c) {
    const int rc = pool_event(g, &gr.region->done[c]);
    if (rc != DS_OK) return rc;
    gr.region->n_done = c + 1;
    W_TRY(hipEventRecord(gr.region->done[c], g->copy_stream[c]));
  }
  gr.region->copies_enqueued = true;
  j.group_begun = false;
  ++j.nc;
  return DS_OK;
}

// the event that says "the whole image is in the host ring"
int finish_job(ds_engine *g, Job &j) {
  ds_event *ev = j.ev;
  W_TRY(hipStreamWaitEvent(g->copy_stream[0], ev->captured, 0));
  if (j.ncs > 1) {
    hipEvent_t tail;
    W_TRY(hipEventCreate(&tail));
    ev->pack_begin.push_back(tail);  // kept only so that it is destroyed with the event
    ev->pack_end.push_back(nullptr);
    W_TRY(hipEventRecord(tail, g->copy_stream[1]));
    W_TRY(hipStreamWaitEvent(g->copy_stream[0], tail, 0));
  }
  if (j.groups.empty()) W_TRY(hipEventRecord(ev->copy_begin, g->copy_stream[0]));
  W_TRY(hipEventRecord(ev->final_ev, g->copy_stream[0]));
  return DS_OK;
}

// The engine thread.  Snapshots are served in the order requested; in every round it (1) takes in new
// requests, (2) issues gathers, oldest snapshot first, for as long as staging has room, (3) issues the
// copies of one more group of the oldest snapshot -- so a gather into a piece of staging is enqueued as soon
// as the copies that last read that piece have been, and with staging as large as what has been requested
// every gather, and with it every gate, is out before the first wait for a ring slot.
void worker_main(ds_engine *g) {
  (void)hipSetDevice(g->device);
  std::deque<Job> active;
  for (;;) {
    int rc = DS_OK;
    try {
      {
        std::unique_lock<std::mutex> lk(g->mu);
        if (active.empty()) g->cv.wait(lk, [&] { return g->stop || !g->queue.empty(); });
        if (active.empty() && g->queue.empty()) return;  // stop requested and nothing left
        while (!g->queue.empty()) {
          active.emplace_back();
          active.back().ev = g->queue.front();
          g->queue.pop_front();
        }
      }
      for (Job &j : active)
        if (!j.prepared && rc == DS_OK) rc = prepare_job(g, j);
      bool room = true;
      for (Job &j : active) {
        while (rc == DS_OK && room && j.np < j.groups.size()) rc = try_issue_pack(g, j, &room);
        if (rc != DS_OK || !room) break;
      }
      if (rc == DS_OK) {
        Job &j = active.front();
        bool blocked = false;
        rc = issue_group_copies(g, j, &blocked);
        if (rc == DS_OK && !blocked && j.nc == j.groups.size() && j.np == j.groups.size()) {
          rc = finish_job(g, j);
          if (rc == DS_OK) {
            {
              std::lock_guard<std::mutex> lk(g->mu);
              j.ev->all_issued = true;
            }
            g->cv.notify_all();
            active.pop_front();
          }
        }
      }
    } catch (const std::bad_alloc &) {
      rc = DS_ENOMEM;
    }
    if (rc != DS_OK) {
      // Issuing failed: every snapshot in hand reports it.  What was enqueued runs out, then staging is
      // taken to be empty.
      (void)hipStreamSynchronize(g->pack_stream);
      for (int c = 0; c < g->n_copy_streams; ++c) (void)hipStreamSynchronize(g->copy_stream[c]);
      forget_regions(g);
      {
        std::lock_guard<std::mutex> lk(g->mu);
        for (Job &j : active) {
          j.ev->error = rc;
          j.ev->all_issued = true;
        }
      }
      g->cv.notify_all();
      active.clear();
    }
  }
}

// waits until the engine thread has enqueued the last gather of this snapshot
int wait_capture_issued(ds_event *ev) {
  ds_engine *g = ev->eng;
  std::unique_lock<std::mutex> lk(g->mu);
  g->cv.wait(lk, [&] { return ev->capture_issued || ev->all_issued; });
  return ev->capture_issued ? DS_OK : ev->error;
}

// waits until the engine thread has issued everything of this snapshot
int wait_issued(ds_event *ev) {
  ds_engine *g = ev->eng;
  std::unique_lock<std::mutex> lk(g->mu);
  g->cv.wait(lk, [&] { return ev->all_issued; });
  return ev->error;
}

void destroy_events(std::vector<hipEvent_t> &v) {
  for (hipEvent_t e : v)
    if (e) (void)hipEventDestroy(e);
  v.clear();
}

void free_engine(ds_engine *g) {
  // the streams are idle here (the callers have synchronised them, or nothing was ever enqueued); they go back
  // to the process's pool in the order they were taken
  for (const PooledStream &ps : g->pooled) stream_give(ps);
  g->pooled.clear();
  forget_regions(g);
  destroy_events(g->event_pool);
  destroy_events(g->ring_done);
  if (g->stage) stage_free(g->device, g->stage, g->stage_cap);
  if (g->ring) ring_free(g->ring, g->ring_cap);
  delete g;
}

}  // namespace

extern "C" {

int ds_engine_create(const ds_engine_opts *o, ds_engine **out) {
  if (!o || !out) return DS_EINVAL;
  if (o->flags & ~(DS_ENGINE_AUTO_RELEASE | DS_ENGINE_TRACE)) return DS_EINVAL;
  const uint64_t chunk = o->d2h_chunk_bytes ? o->d2h_chunk_bytes : (128ull << 20);
  const uint64_t ring_bytes = o->host_ring_bytes ? o->host_ring_bytes : (2ull << 30);
  const uint64_t slot = o->stage_slot_bytes ? o->stage_slot_bytes : (1ull << 30);
  const uint32_t slots = o->stage_slots ? o->stage_slots : 2;
  const uint32_t ncs = o->copy_streams ? o->copy_streams : 1;
  const uint64_t first = o->first_launch_bytes ? o->first_launch_bytes : slot;
  if ((chunk & 4095) || slot % chunk || first % chunk || first > slot || ring_bytes < chunk ||
      ncs > (uint32_t)kMaxCopyStreams || slots > 1024)
    return DS_EINVAL;
  ds_engine *g = new (std::nothrow) ds_engine;
  if (!g) return DS_ENOMEM;
  g->flags = o->flags;
  g->grid_limit = o->pack_grid_limit;
  g->chunk_bytes = chunk;
  g->stage_slot_bytes = slot;
  g->first_launch_bytes = first;
  g->stage_slots = slots;
  g->stage_bytes = slot * slots;
  g->restore_piece_bytes = 8 * chunk < slot ? 8 * chunk : slot;
  g->restore_pieces = (uint32_t)(g->stage_bytes / g->restore_piece_bytes);
  g->ring_slots = (uint32_t)(ring_bytes / chunk);
  g->n_copy_streams = (int)ncs;
  hipError_t e = hipGetDevice(&g->device);
  try {
    for (int k = 0; k < 1 + g->n_copy_streams && e == hipSuccess; ++k) {
      PooledStream ps = {g->device, 0, nullptr};
      e = stream_take(g->device, &ps);
      if (e != hipSuccess) break;
      g->pooled.push_back(ps);
      (k == 0 ? g->pack_stream : g->copy_stream[k - 1]) = ps.stream;
    }
  } catch (const std::bad_alloc &) {
    free_engine(g);
    return DS_ENOMEM;
  }
  if (e == hipSuccess) {
    e = stage_alloc(g->device, slot * slots, &g->stage, &g->stage_cap);
    if (e == hipErrorOutOfMemory) { free_engine(g); return DS_ENOMEM; }
  }
  if (e == hipSuccess) {
    // allocated and pinned once, reused by every snapshot (Sec. V-A1)
    e = ring_alloc((uint64_t)g->ring_slots * chunk, &g->ring, &g->ring_cap);
    if (e == hipErrorOutOfMemory) { free_engine(g); return DS_ENOMEM; }
  }
  try {
    g->ring_done.assign(g->ring_slots, nullptr);
    g->ring_busy.assign(g->ring_slots, 0);
    g->ring_stream.assign(g->ring_slots, -1);
  } catch (const std::bad_alloc &) {
    free_engine(g);
    return DS_ENOMEM;
  }
  for (uint32_t r = 0; r < g->ring_slots && e == hipSuccess; ++r) {
    e = hipEventCreateWithFlags(&g->ring_done[r], hipEventDisableTiming);  // only ever waited for, never timed
    // recorded once so that a wait on a never-used slot is a no-op by construction
    if (e == hipSuccess) e = hipEventRecord(g->ring_done[r], g->copy_stream[0]);
  }
  if (e != hipSuccess) {
    ds_set_hip_error(e);
    free_engine(g);
    return DS_EHIP;
  }
  try {
    g->worker = std::thread(worker_main, g);
  } catch (...) {
    free_engine(g);
    return DS_ENOMEM;
  }
  *out = g;
  return DS_OK;
}

int ds_engine_destroy(ds_engine *g) {
  if (!g) return DS_EINVAL;
  {
    std::lock_guard<std::mutex> lk(g->mu);
    if (g->live_events > 0) return DS_EBUSY;
    g->stop = true;
  }
  g->cv.notify_all();
  if (g->worker.joinable()) g->worker.join();
  int rc = DS_OK;
  hipError_t e = hipStreamSynchronize(g->pack_stream);
  for (int c = 0; c < g->n_copy_streams && e == hipSuccess; ++c) e = hipStreamSynchronize(g->copy_stream[c]);
  if (e != hipSuccess) rc = hip_fail(e);
  free_engine(g);
  return rc;
}

int ds_snapshot_async(ds_engine *g, const ds_plan *plan, void *compute_stream, ds_event **out) {
  if (!g || !plan || !out || !plan->dev_blob) return DS_EINVAL;
  const auto t0 = std::chrono::steady_clock::now();
  {
    std::lock_guard<std::mutex> lk(g->mu);
    if (g->restoring) return DS_EBUSY;
  }
  ds_event *ev = new (std::nothrow) ds_event;
  if (!ev) return DS_ENOMEM;
  ev->eng = g;
  ev->plan = plan;
  try {
    const uint64_t T = plan->total_bytes;
    const uint64_t n = (T + g->chunk_bytes - 1) / g->chunk_bytes;
    ev->chunks.resize(n);
    // chunk boundaries restart at every staging group, so walk the groups
    uint64_t at = 0, k = 0;
    uint32_t group = 0;
    while (at < T) {
      const uint64_t want = group == 0 ? g->first_launch_bytes : g->stage_slot_bytes;
      const uint64_t hi = at + want < T ? at + want : T;
      for (uint64_t lo = at; lo < hi; lo += g->chunk_bytes, ++k) {
        ev->chunks[k].file_off = lo;
        ev->chunks[k].len = lo + g->chunk_bytes < hi ? g->chunk_bytes : hi - lo;
      }
      at = hi;
      ++group;
    }
    ev->chunks.resize(k);
  } catch (const std::bad_alloc &) {
    delete ev;
    return DS_ENOMEM;
  }
  hipError_t e = hipEventCreate(&ev->requested);
  // the point of consistency: everything enqueued so far on the caller's stream
  if (e == hipSuccess) e = hipEventRecord(ev->requested, (hipStream_t)compute_stream);
  if (e != hipSuccess) {
    if (ev->requested) (void)hipEventDestroy(ev->requested);
    delete ev;
    return hip_fail(e);
  }
  {
    std::lock_guard<std::mutex> lk(g->mu);
    g->queue.push_back(ev);
    ++g->live_events;
  }
  g->cv.notify_all();
  ev->submit_host_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
  *out = ev;
  return DS_OK;
}

int ds_event_wait_on_stream(ds_event *ev, void *stream) {
  if (!ev) return DS_EINVAL;
  if (ev->restore) {  // the stream may touch the tensors once the last scatter has run
    {
      // the thread that submits the chunks sets these; the gate may come from another one
      std::lock_guard<std::mutex> lk(ev->eng->mu);
      if (!ev->all_issued) return DS_ESTATE;
      if (ev->error != DS_OK) return ev->error;
    }
    DS_HIP_TRY(hipStreamWaitEvent((hipStream_t)stream, ev->final_ev, 0));
    return DS_OK;
  }
  int rc = wait_capture_issued(ev);
  if (rc != DS_OK) return rc;
  DS_HIP_TRY(hipStreamWaitEvent((hipStream_t)stream, ev->captured, 0));
  return DS_OK;
}

int ds_event_wait_captured(ds_event *ev) {
  if (!ev) return DS_EINVAL;
  if (ev->restore) return DS_ESTATE;
  int rc = wait_capture_issued(ev);
  if (rc != DS_OK) return rc;
  DS_HIP_TRY(hipEventSynchronize(ev->captured));
  return DS_OK;
}

int ds_event_query(ds_event *ev) {
  if (!ev) return DS_EINVAL;
  {
    std::lock_guard<std::mutex> lk(ev->eng->mu);
    if (!ev->all_issued) return DS_NOT_READY;
    if (ev->error != DS_OK) return ev->error;
  }
  hipError_t e = hipEventQuery(ev->final_ev);
  if (e == hipSuccess) return DS_OK;
  if (e == hipErrorNotReady) return DS_NOT_READY;
  return hip_fail(e);
}

int ds_event_wait(ds_event *ev) {
  if (!ev) return DS_EINVAL;
  if (ev->restore) {
    std::lock_guard<std::mutex> lk(ev->eng->mu);
    if (!ev->all_issued) return DS_ESTATE;  // chunks still to be submitted by the caller
  }
  int rc = wait_issued(ev);
  if (rc != DS_OK) return rc;
  DS_HIP_TRY(hipEventSynchronize(ev->final_ev));
  return DS_OK;
}

int ds_snapshot_next_chunk(ds_event *ev, const void **host_ptr, uint64_t *file_off, uint64_t *len) {
  if (!ev || !host_ptr || !file_off || !len) return DS_EINVAL;
  ds_engine *g = ev->eng;
  if ((g->flags & DS_ENGINE_AUTO_RELEASE) || ev->restore) return DS_ESTATE;
  uint32_t k, r;
  {
    std::unique_lock<std::mutex> lk(g->mu);
    if (ev->cursor >= ev->chunks.size()) return DS_EOF;
    k = ev->cursor;
    g->cv.wait(lk, [&] { return ev->chunks[k].state >= 1 || (ev->all_issued && ev->error != DS_OK); });
    if (ev->chunks[k].state < 1) return ev->error;
    r = ev->chunks[k].ring_slot;
  }
  DS_HIP_TRY(hipEventSynchronize(g->ring_done[r]));
  {
    std::lock_guard<std::mutex> lk(g->mu);
    ev->chunks[k].state = 2;
    ev->cursor = k + 1;
  }
  *host_ptr = g->ring + (uint64_t)r * g->chunk_bytes;
  *file_off = ev->chunks[k].file_off;
  *len = ev->chunks[k].len;
  return DS_OK;
}

int ds_snapshot_release_chunk(ds_event *ev, const void *host_ptr) {
  if (!ev || !host_ptr) return DS_EINVAL;
  if (ev->restore) return DS_ESTATE;
  ds_engine *g = ev->eng;
  const uint8_t *p = (const uint8_t *)host_ptr;
  if (p < g->ring || p >= g->ring + (uint64_t)g->ring_slots * g->chunk_bytes || (uint64_t)(p - g->ring) % g->chunk_bytes)
    return DS_ESTATE;
  const uint32_t r = (uint32_t)((uint64_t)(p - g->ring) / g->chunk_bytes);
  {
    std::lock_guard<std::mutex> lk(g->mu);
    DsChunk *hit = nullptr;
    for (uint32_t k = 0; k < ev->cursor && !hit; ++k)
      if (ev->chunks[k].state == 2 && ev->chunks[k].ring_slot == r) hit = &ev->chunks[k];
    if (!hit) return DS_ESTATE;
    hit->state = 3;
    g->ring_busy[r] = 0;
  }
  g->cv.notify_all();
  return DS_OK;
}

int ds_event_stats(ds_event *ev, ds_snapshot_stats *out) {
  if (!ev || !out) return DS_EINVAL;
  int rc = ds_event_query(ev);
  if (rc == DS_NOT_READY) return DS_EBUSY;
  if (rc != DS_OK) return rc;
  out->image_bytes = ev->plan->total_bytes;
  out->payload_bytes = ev->plan->payload_bytes;
  out->n_copies = (uint32_t)ev->chunks.size();
  out->n_pack_launches = 0;
  out->pack_ms = 0;
  for (size_t i = 0; i < ev->pack_begin.size(); ++i) {
    if (!ev->pack_end[i]) continue;
    float ms = 0;
    DS_HIP_TRY(hipEventElapsedTime(&ms, ev->pack_begin[i], ev->pack_end[i]));
    out->pack_ms += ms;
    ++out->n_pack_launches;
  }
  float ms = 0;
  DS_HIP_TRY(hipEventElapsedTime(&ms, ev->copy_begin, ev->final_ev));
  out->copy_ms = ms;
  if (ev->captured) DS_HIP_TRY(hipEventElapsedTime(&ms, ev->requested, ev->captured));
  out->capture_ms = ev->captured ? ms : 0.0;
  DS_HIP_TRY(hipEventElapsedTime(&ms, ev->requested, ev->final_ev));
  out->total_ms = ms;
  out->submit_host_ms = ev->submit_host_ms;
  return DS_OK;
}

int ds_event_trace(ds_event *ev, ds_trace_rec *out, size_t cap, size_t *n) {
  if (!ev || !n || (!out && cap)) return DS_EINVAL;
  if (ev->restore) return DS_ESTATE;
  int rc = ds_event_query(ev);
  if (rc == DS_NOT_READY) return DS_EBUSY;
  if (rc != DS_OK) return rc;
  size_t k = 0;
  auto put = [&](uint32_t kind, uint32_t index, uint64_t off, uint64_t len, hipEvent_t b, hipEvent_t e) -> int {
    if (k < cap) {
      float tb = 0, te = 0;
      DS_HIP_TRY(hipEventElapsedTime(&tb, ev->requested, b));
      DS_HIP_TRY(hipEventElapsedTime(&te, ev->requested, e));
      out[k] = {kind, index, off, len, (double)tb, (double)te};
    }
    ++k;
    return DS_OK;
  };
  for (size_t i = 0; i < ev->pack_lo.size(); ++i) {
    rc = put(0, (uint32_t)i, ev->pack_lo[i], ev->pack_hi[i] - ev->pack_lo[i], ev->pack_begin[i], ev->pack_end[i]);
    if (rc != DS_OK) return rc;
  }
  for (size_t i = 0; i < ev->copy_b.size() && i < ev->copy_e.size(); ++i) {
    rc = put(1, (uint32_t)i, ev->chunks[i].file_off, ev->chunks[i].len, ev->copy_b[i], ev->copy_e[i]);
    if (rc != DS_OK) return rc;
  }
  *n = k;
  return DS_OK;
}

int ds_event_destroy(ds_event *ev) {
  if (!ev) return DS_EINVAL;
  ds_engine *g = ev->eng;
  int rc = DS_OK;
  if (ev->restore) {
    // whatever was submitted runs to its end; chunks never submitted are simply not restored
    hipError_t e = hipSuccess;
    for (int c = 0; c < g->n_copy_streams && e == hipSuccess; ++c) e = hipStreamSynchronize(g->copy_stream[c]);
    if (e == hipSuccess) e = hipStreamSynchronize(g->pack_stream);
    if (e != hipSuccess) rc = hip_fail(e);
    destroy_events(ev->group_done);
    destroy_events(ev->pack_begin);
    destroy_events(ev->pack_end);
    for (hipEvent_t x : {ev->requested, ev->captured, ev->final_ev, ev->copy_begin})
      if (x) (void)hipEventDestroy(x);
    {
      std::lock_guard<std::mutex> lk(g->mu);
      std::fill(g->ring_busy.begin(), g->ring_busy.end(), 0);  // the ring is empty again for snapshots
      --g->live_events;
      g->restoring = false;
    }
    delete ev;
    return rc;
  }
  if (!(g->flags & DS_ENGINE_AUTO_RELEASE)) {
    // hand back what the consumer still holds, then drain what it never took
    for (;;) {
      const void *p = nullptr;
      {
        std::lock_guard<std::mutex> lk(g->mu);
        for (uint32_t k = 0; k < ev->cursor && !p; ++k)
          if (ev->chunks[k].state == 2) p = g->ring + (uint64_t)ev->chunks[k].ring_slot * g->chunk_bytes;
      }
      if (!p) break;
      (void)ds_snapshot_release_chunk(ev, p);
    }
    for (;;) {
      const void *p;
      uint64_t off, len;
      int r = ds_snapshot_next_chunk(ev, &p, &off, &len);
      if (r != DS_OK) break;
      (void)ds_snapshot_release_chunk(ev, p);
    }
  }
  int w = wait_issued(ev);
  if (w == DS_OK && ev->final_ev) {
    hipError_t e = hipEventSynchronize(ev->final_ev);
    if (e != hipSuccess) rc = hip_fail(e);
  } else if (w != DS_OK) {
    // issuing failed half-way: make sure nothing of it is still running
    (void)hipStreamSynchronize(g->pack_stream);
    for (int c = 0; c < g->n_copy_streams; ++c) (void)hipStreamSynchronize(g->copy_stream[c]);
  }
  destroy_events(ev->pack_begin);
  destroy_events(ev->pack_end);
  destroy_events(ev->copy_b);
  destroy_events(ev->copy_e);
  for (hipEvent_t e : {ev->requested, ev->captured, ev->final_ev, ev->copy_begin})
    if (e) (void)hipEventDestroy(e);
  {
    std::lock_guard<std::mutex> lk(g->mu);
    --g->live_events;
  }
  delete ev;
  return rc;
}


// ---- restore: pinned host ring -> device staging -> scatter (the mirror image of a snapshot) -----

int ds_restore_begin(ds_engine *g, const ds_plan *plan, void *compute_stream, ds_event **out) {
  if (!g || !plan || !out || !plan->dev_blob) return DS_EINVAL;
  {
    std::lock_guard<std::mutex> lk(g->mu);
    if (g->live_events > 0) return DS_EBUSY;  // ring and staging are shared with snapshots
    ++g->live_events;
    g->restoring = true;
  }
  ds_event *ev = new (std::nothrow) ds_event;
  int rc = ev ? DS_OK : DS_ENOMEM;
  hipError_t e = hipSuccess;
  if (rc == DS_OK) {
    ev->eng = g;
    ev->plan = plan;
    ev->restore = true;
    try {
      const uint64_t T = plan->total_bytes;
      for (uint64_t lo = 0; lo < T; lo += g->chunk_bytes) {
        DsChunk c;
        c.file_off = lo;
        c.len = lo + g->chunk_bytes < T ? g->chunk_bytes : T - lo;
        ev->chunks.push_back(c);
      }
      ev->group_done.assign((size_t)((T + g->restore_piece_bytes - 1) / g->restore_piece_bytes), nullptr);
    } catch (const std::bad_alloc &) {
      rc = DS_ENOMEM;
    }
  }
  if (rc == DS_OK) {
    // the engine is idle by contract; make sure its streams are, so that slots and staging are free
    e = hipStreamSynchronize(g->pack_stream);
    for (int c = 0; c < g->n_copy_streams && e == hipSuccess; ++c) e = hipStreamSynchronize(g->copy_stream[c]);
    if (e == hipSuccess) forget_regions(g);  // nothing reads staging any more; the restore lays it out in slots
    if (e == hipSuccess) e = hipEventCreate(&ev->requested);
    if (e == hipSuccess) e = hipEventCreate(&ev->final_ev);
    if (e == hipSuccess) e = hipEventCreate(&ev->copy_begin);
    for (size_t i = 0; i < ev->group_done.size() && e == hipSuccess; ++i) e = hipEventCreate(&ev->group_done[i]);
    // scatters must not start before what the caller has enqueued so far on its stream
    if (e == hipSuccess) e = hipEventRecord(ev->requested, (hipStream_t)compute_stream);
    if (e == hipSuccess) e = hipStreamWaitEvent(g->pack_stream, ev->requested, 0);
    if (e == hipSuccess) e = hipEventRecord(ev->copy_begin, g->copy_stream[0]);
    if (e == hipSuccess && ev->chunks.empty()) {
      e = hipEventRecord(ev->final_ev, g->pack_stream);
      ev->all_issued = ev->capture_issued = true;
    }
    if (e != hipSuccess) rc = hip_fail(e);
  }
  if (rc != DS_OK) {
    if (ev) {
      destroy_events(ev->group_done);
      for (hipEvent_t x : {ev->requested, ev->final_ev, ev->copy_begin})
        if (x) (void)hipEventDestroy(x);
      delete ev;
    }
    std::lock_guard<std::mutex> lk(g->mu);
    --g->live_events;
    g->restoring = false;
    return rc;
  }
  std::fill(g->ring_busy.begin(), g->ring_busy.end(), 0);
  std::fill(g->ring_stream.begin(), g->ring_stream.end(), (int8_t)-1);  // the copy streams are idle: no slot needs a wait
  *out = ev;
  return DS_OK;
}

int ds_restore_next_slot(ds_event *ev, void **host_ptr, uint64_t *file_off, uint64_t *len) {
  if (!ev || !host_ptr || !file_off || !len) return DS_EINVAL;
  if (!ev->restore) return DS_ESTATE;
  ds_engine *g = ev->eng;
  if (ev->r_handed >= ev->chunks.size()) return DS_EOF;
  if (ev->r_handed - ev->r_submitted >= g->ring_slots) return DS_EBUSY;  // every slot is with the caller
  const uint32_t k = ev->r_handed;
  const uint32_t r = k % g->ring_slots;
  // the slot's previous content must have left for the device
  if (g->ring_busy[r]) DS_HIP_TRY(hipEventSynchronize(g->ring_done[r]));
  ev->chunks[k].ring_slot = r;
  ev->chunks[k].state = 2;
  ev->r_handed = k + 1;
  *host_ptr = g->ring + (uint64_t)r * g->chunk_bytes;
  *file_off = ev->chunks[k].file_off;
  *len = ev->chunks[k].len;
  return DS_OK;
}

int ds_restore_submit(ds_event *ev, const void *host_ptr) {
  if (!ev || !host_ptr) return DS_EINVAL;
  if (!ev->restore) return DS_ESTATE;
  ds_engine *g = ev->eng;
  const uint32_t k = ev->r_submitted;  // chunks are submitted in the order they were handed out
  if (k >= ev->r_handed) return DS_ESTATE;
  DsChunk &c = ev->chunks[k];
  if (host_ptr != g->ring + (uint64_t)c.ring_slot * g->chunk_bytes) return DS_ESTATE;
  const uint64_t S = g->restore_piece_bytes;
  const size_t gi = (size_t)(c.file_off / S);
  const uint64_t glo = (uint64_t)gi * S;
  const uint64_t ghi = glo + S < ev->plan->total_bytes ? glo + S : ev->plan->total_bytes;
  const uint32_t s = (uint32_t)(gi % g->restore_pieces);
  uint8_t *slot = g->stage + (uint64_t)s * S;
  // chunks alternate over the copy streams, as in a snapshot
  hipStream_t cs = g->copy_stream[k % (uint32_t)g->n_copy_streams];
  // the staging slot must have been scattered out by the group that used it before (a wait per chunk:
  // either stream may carry the group's first chunk; it costs nothing once the event has fired)
  if (gi >= g->restore_pieces) W_TRY(hipStreamWaitEvent(cs, ev->group_done[gi - g->restore_pieces], 0));
  W_TRY(hipMemcpyAsync(slot + (c.file_off - glo), host_ptr, c.len, hipMemcpyHostToDevice, cs));
  W_TRY(hipEventRecord(g->ring_done[c.ring_slot], cs));
  g->ring_busy[c.ring_slot] = 1;
  c.state = 3;
  ev->r_submitted = k + 1;
  if (c.file_off + c.len == ghi) {  // the group is complete: scatter it
    hipEvent_t b, e;
    W_TRY(hipEventCreate(&b));
    ev->pack_begin.push_back(b);
    W_TRY(hipEventCreate(&e));
    ev->pack_end.push_back(e);
    // every copy of the group has landed: the last one, and the one before it, which is the last one of
    // the other copy stream (each stream runs its copies in order)
    W_TRY(hipStreamWaitEvent(g->pack_stream, g->ring_done[c.ring_slot], 0));
    if (g->n_copy_streams > 1 && k > 0)
      W_TRY(hipStreamWaitEvent(g->pack_stream, g->ring_done[ev->chunks[k - 1].ring_slot], 0));
    W_TRY(hipEventRecord(b, g->pack_stream));
    int rc = ds_launch_move(ev->plan, false, slot, glo, ghi, g->grid_limit, g->pack_stream);
    if (rc != DS_OK) return rc;
    W_TRY(hipEventRecord(e, g->pack_stream));
    W_TRY(hipEventRecord(ev->group_done[gi], g->pack_stream));
    if (ghi == ev->plan->total_bytes) {
      W_TRY(hipEventRecord(ev->final_ev, g->pack_stream));
      std::lock_guard<std::mutex> lk(g->mu);
      ev->all_issued = ev->capture_issued = true;
    }
  }
  return DS_OK;
}

}  // extern "C"
