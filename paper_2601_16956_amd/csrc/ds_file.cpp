// Host <-> file tier of the snapshot pipeline (DataStates-LLM Sec. V-A4: a
// chunk moves on to the next tier as soon as it is resident; Sec. V-C: file
// persistence runs on background threads in native code, with direct I/O).
//
// Built on the public chunk interface only: a flush is a consumer of
// ds_snapshot_next_chunk / ds_snapshot_release_chunk, a file restore is a
// producer for ds_restore_next_slot / ds_restore_submit.  Writes and reads go
// to the byte offsets the plan fixed (Sec. V-A5 rule (1)), so several threads
// work on one file without coordination.  Writes go out either from a pool of
// threads that call pwrite, or -- DS_FILE_URING -- from ONE thread that keeps
// up to `threads` writes in flight through the kernel's io_uring interface
// (Sec. V-C names liburing; that library is not installed here, so the rings
// are set up and driven with the raw system calls).  Reads use pread threads.
#include <fcntl.h>
#include <linux/io_uring.h>
#include <sys/mman.h>
#include <sys/stat.h>
#include <sys/syscall.h>
#include <unistd.h>

#include <algorithm>
#include <atomic>
#include <cerrno>
#include <cstdlib>
#include <cstring>
#include <chrono>
#include <condition_variable>
#include <deque>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

#include "ds_internal.h"

namespace {

thread_local int g_last_errno = 0;

// A ring slot that one or more writes read from: it goes back to the snapshot when the last of them is done
// with it.  A chunk that spans the boundary between two files is written as two pieces.
struct Held {
  void *ptr = nullptr;
  std::atomic<int> left{0};
};

struct IoJob {
  void *ptr = nullptr;          // memory of this piece
  uint64_t off = 0, len = 0;    // where it goes in (comes from) its file
  int slot = -1;                // restore: index into the in-flight window
  uint32_t target = 0;          // which file
  Held *held = nullptr;         // flush: the ring slot the piece lies in
};

// Cuts image range [off, off + len) at the boundaries of the files and calls piece(target, offset in that
// file, offset in the range, length) for every non-empty part.  The targets are in image order and cover
// the image without holes; the last one is open-ended for a caller that does not know the image length.
template <class F>
void for_each_piece(const std::vector<DsFileTarget> &targets, uint64_t off, uint64_t len, F piece) {
  size_t t = 0;
  while (t + 1 < targets.size() && targets[t].end <= off) ++t;
  uint64_t at = off;
  const uint64_t stop = off + len;
  while (at < stop && t < targets.size()) {
    const uint64_t e = std::min(stop, targets[t].end);
    if (e > at) {
      piece((uint32_t)t, at - targets[t].begin, at - off, e - at);
      at = e;
    }
    if (at < stop) ++t;
  }
}

bool direct_ok(const void *p, uint64_t off, uint64_t len) {
  return (((uintptr_t)p | off | len) & 4095) == 0;
}

// whole-range pwrite / pread; returns 0 or errno
int write_all(int fd, const uint8_t *p, uint64_t len, uint64_t off) {
  while (len) {
    ssize_t w = pwrite(fd, p, len, (off_t)off);
    if (w < 0) {
      if (errno == EINTR) continue;
      return errno;
    }
    p += w;
    off += (uint64_t)w;
    len -= (uint64_t)w;
  }
  return 0;
}
int read_all(int fd, uint8_t *p, uint64_t len, uint64_t off) {
  while (len) {
    ssize_t r = pread(fd, p, len, (off_t)off);
    if (r < 0) {
      if (errno == EINTR) continue;
      return errno;
    }
    if (r == 0) return EIO;  // file shorter than the image
    p += r;
    off += (uint64_t)r;
    len -= (uint64_t)r;
  }
  return 0;
}

double now_s() {
  return std::chrono::duration<double>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

}  // namespace

struct ds_flush {
  ds_event *ev = nullptr;
  std::vector<DsFileTarget> targets;  // the files, in image order
  uint32_t flags = 0;
  bool own_fds = true;  // false: the descriptors belong to checkpoint writers, which sync and close them
  std::thread dispatcher;
  std::vector<std::thread> writers;
  std::mutex mu;
  std::condition_variable cv;
  std::deque<IoJob> queue;
  bool no_more = false;
  std::atomic<int> status{DS_OK};
  std::atomic<int> err_no{0};
  std::atomic<uint64_t> bytes{0};
  std::atomic<bool> direct_usable{true};  // direct I/O straight from the ring's pages
  std::atomic<bool> bounce_usable{true};  // direct I/O from a copy in ordinary memory
  double t0 = 0, t1 = 0;
};

namespace {

void flush_fail(ds_flush *f, int status, int e) {
  int expect = DS_OK;
  if (f->status.compare_exchange_strong(expect, status)) f->err_no.store(e);
}

// This piece no longer needs its ring slot; the last piece of a slot hands it back.
void release_piece(ds_flush *f, const IoJob &j) {
  if (j.held->left.fetch_sub(1) != 1) return;
  int rc = ds_snapshot_release_chunk(f->ev, j.held->ptr);
  if (rc != DS_OK) flush_fail(f, rc, 0);
  delete j.held;
}

// A 4 KiB-aligned buffer of ordinary memory, grown on demand: direct I/O cannot take the pinned ring's pages
// (the kernel refuses to pin them a second time), so a slot is copied here first -- one memory-speed copy
// instead of a trip through the page cache.
struct Bounce {
  uint8_t *p = nullptr;
  uint64_t cap = 0;
  ~Bounce() { free(p); }
  uint8_t *fit(uint64_t n) {
    if (n > cap) {
      free(p);
      p = nullptr;
      cap = 0;
      void *q = nullptr;
      if (posix_memalign(&q, 4096, (size_t)n) != 0) return nullptr;
      p = (uint8_t *)q;
      cap = n;
    }
    return p;
  }
};

void writer_main(ds_flush *f) {
  Bounce bounce;
  for (;;) {
    IoJob j;
    {
      std::unique_lock<std::mutex> lk(f->mu);
      f->cv.wait(lk, [&] { return f->no_more || !f->queue.empty(); });
      if (f->queue.empty()) return;
      j = f->queue.front();
      f->queue.pop_front();
    }
    bool released = false;
    if (f->status.load() == DS_OK) {
      const int fd_direct = f->targets[j.target].fd_direct, fd_buffered = f->targets[j.target].fd_buffered;
      const bool direct = fd_direct >= 0 && direct_ok(j.ptr, j.off, j.len);
      int e = -1;  // -1: not written yet, try the next way
      if (direct && f->direct_usable.load()) {           // straight from the ring, where the kernel allows it
        e = write_all(fd_direct, (const uint8_t *)j.ptr, j.len, j.off);
        if (e == EFAULT || e == EINVAL) {
          f->direct_usable.store(false);
          e = -1;
        }
      }
      if (e == -1 && direct && f->bounce_usable.load()) {  // through an aligned buffer of ordinary memory
        uint8_t *b = bounce.fit(j.len);
        if (b) {
          std::memcpy(b, j.ptr, j.len);
          // the copy is what the file gets: the ring slot is free for the next device-to-host copy already
          release_piece(f, j);
          released = true;
          e = write_all(fd_direct, b, j.len, j.off);
          if (e == EINVAL) {                             // the file system has no direct I/O after all
            f->bounce_usable.store(false);
            e = write_all(fd_buffered, b, j.len, j.off);
          }
        }
      }
      if (e == -1) e = write_all(fd_buffered, (const uint8_t *)j.ptr, j.len, j.off);
      if (e) flush_fail(f, DS_EIO, e);
      else f->bytes.fetch_add(j.len);
    }
    // the slot goes back whatever happened, so that the snapshot itself can finish
    if (!released) release_piece(f, j);
  }
}

// ---- io_uring, by system call ---------------------------------------------------------------
// The submission ring holds indices into an array of request entries, the completion ring the results;
// both are shared with the kernel and updated with acquire / release accesses to their head and tail.
struct Uring {
  int fd = -1;
  unsigned entries = 0, pending = 0, tail_local = 0;
  unsigned *sq_head = nullptr, *sq_tail = nullptr, *sq_mask = nullptr, *sq_array = nullptr;
  unsigned *cq_head = nullptr, *cq_tail = nullptr, *cq_mask = nullptr;
  io_uring_sqe *sqes = nullptr;
  io_uring_cqe *cqes = nullptr;
  void *sq_map = MAP_FAILED, *cq_map = MAP_FAILED, *sqe_map = MAP_FAILED;
  size_t sq_len = 0, cq_len = 0, sqe_len = 0;

  int open_ring(unsigned want) {  // 0 or errno
    io_uring_params p;
    std::memset(&p, 0, sizeof(p));
    fd = (int)syscall(__NR_io_uring_setup, want, &p);
    if (fd < 0) return errno;
    sq_len = p.sq_off.array + p.sq_entries * sizeof(unsigned);
    cq_len = p.cq_off.cqes + p.cq_entries * sizeof(io_uring_cqe);
    const bool single = (p.features & IORING_FEAT_SINGLE_MMAP) != 0;
    if (single) sq_len = cq_len = std::max(sq_len, cq_len);
    sq_map = mmap(nullptr, sq_len, PROT_READ | PROT_WRITE, MAP_SHARED | MAP_POPULATE, fd, IORING_OFF_SQ_RING);
    if (sq_map == MAP_FAILED) return errno ? errno : ENOMEM;
    cq_map = single ? sq_map
                    : mmap(nullptr, cq_len, PROT_READ | PROT_WRITE, MAP_SHARED | MAP_POPULATE, fd, IORING_OFF_CQ_RING);
    if (cq_map == MAP_FAILED) return errno ? errno : ENOMEM;
    sqe_len = p.sq_entries * sizeof(io_uring_sqe);
    sqe_map = mmap(nullptr, sqe_len, PROT_READ | PROT_WRITE, MAP_SHARED | MAP_POPULATE, fd, IORING_OFF_SQES);
    if (sqe_map == MAP_FAILED) return errno ? errno : ENOMEM;
    uint8_t *sq = (uint8_t *)sq_map, *cq = (uint8_t *)cq_map;
    sq_head = (unsigned *)(sq + p.sq_off.head);
    sq_tail = (unsigned *)(sq + p.sq_off.tail);
    sq_mask = (unsigned *)(sq + p.sq_off.ring_mask);
    sq_array = (unsigned *)(sq + p.sq_off.array);
    cq_head = (unsigned *)(cq + p.cq_off.head);
    cq_tail = (unsigned *)(cq + p.cq_off.tail);
    cq_mask = (unsigned *)(cq + p.cq_off.ring_mask);
    cqes = (io_uring_cqe *)(cq + p.cq_off.cqes);
    sqes = (io_uring_sqe *)sqe_map;
    entries = p.sq_entries;
    tail_local = *sq_tail;
    return 0;
  }
  void close_ring() {
    if (sqe_map != MAP_FAILED) munmap(sqe_map, sqe_len);
    if (cq_map != MAP_FAILED && cq_map != sq_map) munmap(cq_map, cq_len);
    if (sq_map != MAP_FAILED) munmap(sq_map, sq_len);
    if (fd >= 0) close(fd);
    sqe_map = cq_map = sq_map = MAP_FAILED;
    fd = -1;
  }
  // queues one write; false if the submission ring is full
  bool queue_write(int file, const void *buf, uint64_t len, uint64_t off, uint64_t user) {
    const unsigned head = __atomic_load_n(sq_head, __ATOMIC_ACQUIRE);
    if (tail_local - head >= entries) return false;
    const unsigned idx = tail_local & *sq_mask;
    io_uring_sqe *e = &sqes[idx];
    std::memset(e, 0, sizeof(*e));
    e->opcode = IORING_OP_WRITE;
    e->fd = file;
    e->addr = (uint64_t)(uintptr_t)buf;
    e->len = (uint32_t)len;
    e->off = off;
    e->user_data = user;
    sq_array[idx] = idx;
    ++tail_local;
    ++pending;
    return true;
  }
  // hands the queued requests to the kernel and waits for at least min_complete results; 0 or errno
  int submit_and_wait(unsigned min_complete) {
    __atomic_store_n(sq_tail, tail_local, __ATOMIC_RELEASE);
    for (;;) {
      const long r = syscall(__NR_io_uring_enter, fd, pending, min_complete, IORING_ENTER_GETEVENTS, nullptr, 0);
      if (r < 0) {
        if (errno == EINTR) continue;
        return errno;
      }
      pending -= (unsigned)r < pending ? (unsigned)r : pending;
      return 0;
    }
  }
  bool pop(uint64_t *user, int *res) {
    const unsigned head = *cq_head;
    if (head == __atomic_load_n(cq_tail, __ATOMIC_ACQUIRE)) return false;
    const io_uring_cqe &c = cqes[head & *cq_mask];
    *user = c.user_data;
    *res = c.res;
    __atomic_store_n(cq_head, head + 1, __ATOMIC_RELEASE);
    return true;
  }
};

constexpr uint64_t kUringMaxWrite = 1u << 30;  // one request carries a 32-bit length

// One thread, up to `depth` writes in flight.  With direct I/O a slot is copied into an aligned buffer of
// ordinary memory and given back to the ring at once; a buffered write goes out of the slot itself, which
// is given back when the write has completed.
void uring_writer_main(ds_flush *f, Uring *ring, unsigned depth) {
  struct Op {
    bool busy = false, direct = false, holds_slot = false;
    IoJob j;
    Bounce bounce;
    const uint8_t *src = nullptr;
    uint64_t off = 0, left = 0;
  };
  std::vector<Op> ops(depth);
  unsigned inflight = 0;
  auto release = [&](Op &op) {
    if (op.holds_slot) {
      release_piece(f, op.j);
      op.holds_slot = false;
    }
  };
  auto queue_op = [&](unsigned i) {
    Op &op = ops[i];
    const uint64_t n = op.left < kUringMaxWrite ? op.left : kUringMaxWrite;
    // the ring has 2 x depth entries and at most depth requests are ever queued: this cannot fail
    const DsFileTarget &t = f->targets[op.j.target];
    (void)ring->queue_write(op.direct ? t.fd_direct : t.fd_buffered, op.src, n, op.off, i);
  };
  for (;;) {
    // take new jobs while there is room
    while (inflight < depth) {
      IoJob j;
      {
        std::unique_lock<std::mutex> lk(f->mu);
        if (inflight == 0) f->cv.wait(lk, [&] { return f->no_more || !f->queue.empty(); });
        if (f->queue.empty()) break;
        j = f->queue.front();
        f->queue.pop_front();
      }
      unsigned i = 0;
      while (ops[i].busy) ++i;
      Op &op = ops[i];
      op.j = j;
      op.holds_slot = true;
      if (f->status.load() != DS_OK) {  // after a failure the slots only go back
        release(op);
        continue;
      }
      op.direct = f->targets[j.target].fd_direct >= 0 && f->bounce_usable.load() && direct_ok(j.ptr, j.off, j.len);
      uint8_t *b = op.direct ? op.bounce.fit(j.len) : nullptr;
      if (op.direct && !b) op.direct = false;
      if (op.direct) {
        std::memcpy(b, j.ptr, j.len);
        release(op);  // the ring slot is free for the next copy while this write is under way
        op.src = b;
      } else {
        op.src = (const uint8_t *)j.ptr;
      }
      op.off = j.off;
      op.left = j.len;
      op.busy = true;
      ++inflight;
      queue_op(i);
    }
    if (inflight == 0) {
      std::lock_guard<std::mutex> lk(f->mu);
      if (f->no_more && f->queue.empty()) break;
      continue;
    }
    const int e = ring->submit_and_wait(1);
    if (e) {  // the interface itself failed: give everything back and stop
      flush_fail(f, DS_EIO, e);
      for (Op &op : ops)
        if (op.busy) release(op);
      for (;;) {
        IoJob j;
        {
          std::unique_lock<std::mutex> lk(f->mu);
          f->cv.wait(lk, [&] { return f->no_more || !f->queue.empty(); });
          if (f->queue.empty()) break;
          j = f->queue.front();
          f->queue.pop_front();
        }
        release_piece(f, j);
      }
      break;
    }
    uint64_t user;
    int res;
    while (ring->pop(&user, &res)) {
      Op &op = ops[(unsigned)user];
      if (res < 0 && op.direct && res == -EINVAL) {
        // the file system has no direct I/O after all: the same bytes through the buffered descriptor
        f->bounce_usable.store(false);
        op.direct = false;
        queue_op((unsigned)user);
        continue;
      }
      if (res == -EAGAIN || res == -EINTR) {  // not an error: the same request once more
        queue_op((unsigned)user);
        continue;
      }
      if (res < 0 || res == 0) {
        flush_fail(f, DS_EIO, res < 0 ? -res : EIO);
      } else if ((uint64_t)res < op.left) {  // a short write: the rest goes out as a new request
        op.src += res;
        op.off += (uint64_t)res;
        op.left -= (uint64_t)res;
        queue_op((unsigned)user);
        continue;
      } else {
        f->bytes.fetch_add(op.j.len);
      }
      release(op);
      op.busy = false;
      --inflight;
    }
  }
  ring->close_ring();
  delete ring;
}

void dispatcher_main(ds_flush *f) {
  for (;;) {
    const void *p = nullptr;
    uint64_t off = 0, len = 0;
    int rc = ds_snapshot_next_chunk(f->ev, &p, &off, &len);
    if (rc == DS_EOF) break;
    if (rc != DS_OK) {
      flush_fail(f, rc, 0);
      break;
    }
    int pieces = 0;
    for_each_piece(f->targets, off, len, [&](uint32_t, uint64_t, uint64_t, uint64_t) { ++pieces; });
    Held *held = pieces ? new (std::nothrow) Held : nullptr;
    if (!held) {  // nothing to write (no file covers the range) or no memory: the slot goes straight back
      if (pieces) flush_fail(f, DS_ENOMEM, 0);
      rc = ds_snapshot_release_chunk(f->ev, const_cast<void *>(p));
      if (rc != DS_OK) flush_fail(f, rc, 0);
      continue;
    }
    held->ptr = const_cast<void *>(p);
    held->left.store(pieces);
    {
      std::lock_guard<std::mutex> lk(f->mu);
      try {
        for_each_piece(f->targets, off, len, [&](uint32_t t, uint64_t file_off, uint64_t in_chunk, uint64_t n) {
          IoJob j;
          j.ptr = (uint8_t *)held->ptr + in_chunk;
          j.off = file_off;
          j.len = n;
          j.target = t;
          j.held = held;
          f->queue.push_back(j);
          --pieces;
        });
      } catch (const std::bad_alloc &) {
        flush_fail(f, DS_ENOMEM, 0);
      }
    }
    // pieces that could not be queued give their share of the slot back here
    for (; pieces > 0; --pieces) {
      IoJob j;
      j.held = held;
      release_piece(f, j);
    }
    f->cv.notify_all();
  }
  {
    std::lock_guard<std::mutex> lk(f->mu);
    f->no_more = true;
  }
  f->cv.notify_all();
}

}  // namespace

int ds_flush_start_fds(ds_event *ev, int fd_buffered, int fd_direct, uint32_t threads, uint32_t flags,
                       ds_flush **out) {
  DsFileTarget t;
  t.begin = 0;
  t.end = ~(uint64_t)0;
  t.fd_buffered = fd_buffered;
  t.fd_direct = fd_direct;
  try {
    return ds_flush_start_targets(ev, std::vector<DsFileTarget>(1, t), threads, flags, out);
  } catch (const std::bad_alloc &) {
    return DS_ENOMEM;
  }
}

int ds_flush_start_targets(ds_event *ev, std::vector<DsFileTarget> targets, uint32_t threads, uint32_t flags,
                           ds_flush **out) {
  if (!ev || !out || targets.empty() || (flags & ~(DS_FILE_DIRECT | DS_FILE_SYNC | DS_FILE_URING))) return DS_EINVAL;
  for (size_t t = 0; t < targets.size(); ++t)
    if (targets[t].fd_buffered < 0 || targets[t].end < targets[t].begin ||
        targets[t].begin != (t ? targets[t - 1].end : 0))
      return DS_EINVAL;
  if (threads == 0) threads = 4;
  if (threads > 64) return DS_EINVAL;
  ds_flush *f = new (std::nothrow) ds_flush;
  if (!f) return DS_ENOMEM;
  f->targets.swap(targets);
  // io_uring if asked for and the kernel lets this process have it; else the pwrite threads
  Uring *ring = nullptr;
  if (flags & DS_FILE_URING) {
    ring = new (std::nothrow) Uring;
    if (ring && ring->open_ring(2 * threads) != 0) {
      ring->close_ring();
      delete ring;
      ring = nullptr;
    }
  }
  f->ev = ev;
  f->flags = flags;
  f->own_fds = false;
  f->t0 = now_s();
  // writers first: a dispatcher without anyone to release slots would wait for ever
  try {
    if (ring) {
      f->writers.emplace_back(uring_writer_main, f, ring, threads);
      ring = nullptr;  // the thread owns it now
    } else {
      for (uint32_t i = 0; i < threads; ++i) f->writers.emplace_back(writer_main, f);
    }
  } catch (...) {
  }
  if (ring) {
    ring->close_ring();
    delete ring;
  }
  bool started = !f->writers.empty();
  if (started) {
    try {
      f->dispatcher = std::thread(dispatcher_main, f);
    } catch (...) {
      started = false;
    }
  }
  if (!started) {
    {
      std::lock_guard<std::mutex> lk(f->mu);
      f->no_more = true;
    }
    f->cv.notify_all();
    for (std::thread &t : f->writers) t.join();
    delete f;
    return DS_ENOMEM;
  }
  *out = f;
  return DS_OK;
}

// The files' descriptors stay the caller's.  Ring slots are read by `threads` readers at once, a slot that
// spans two files in two pieces, and submitted in image order.
int ds_restore_from_targets(ds_engine *engine, const ds_plan *plan, const std::vector<DsFileTarget> &targets,
                            uint32_t threads, void *compute_stream, ds_event **out) {
  if (!engine || !plan || !out || targets.empty()) return DS_EINVAL;
  if (threads == 0) threads = 4;
  if (threads > 64) return DS_EINVAL;
  for (size_t t = 0; t < targets.size(); ++t)
    if (targets[t].fd_buffered < 0 || targets[t].end < targets[t].begin ||
        targets[t].begin != (t ? targets[t - 1].end : 0))
      return DS_EINVAL;
  if (targets.back().end < plan->total_bytes) return DS_EINVAL;
  ds_event *ev = nullptr;
  int rc = ds_restore_begin(engine, plan, compute_stream, &ev);
  if (rc != DS_OK) return rc;
  struct Shared {
    std::mutex mu;
    std::condition_variable cv;
    std::deque<IoJob> todo;
    std::vector<int> done;  // per window position: 0 pending, 1 read, <0 = -errno
    std::vector<int> left;  // pieces of that slot still being read
    bool stop = false;
  } sh;
  std::atomic<bool> direct_usable{true}, bounce_usable{true};
  const uint32_t window = 2 * threads;  // slots beyond the readers, so that one slow read does not idle the others
  sh.done.assign(window, 0);
  sh.left.assign(window, 0);
  std::vector<void *> win(window);  // the slot at each window position
  std::vector<std::thread> readers;
  auto reader = [&]() {
    Bounce bounce;
    for (;;) {
      IoJob j;
      {
        std::unique_lock<std::mutex> lk(sh.mu);
        sh.cv.wait(lk, [&] { return sh.stop || !sh.todo.empty(); });
        if (sh.todo.empty()) return;
        j = sh.todo.front();
        sh.todo.pop_front();
      }
      // the same three ways as in writer_main: direct into the ring, direct into an aligned buffer of
      // ordinary memory and a copy, buffered
      const int fd_direct = targets[j.target].fd_direct, fd_buffered = targets[j.target].fd_buffered;
      const bool direct = fd_direct >= 0 && direct_ok(j.ptr, j.off, j.len);
      int e = -1;
      if (direct && direct_usable.load()) {
        e = read_all(fd_direct, (uint8_t *)j.ptr, j.len, j.off);
        if (e == EFAULT || e == EINVAL) {
          direct_usable.store(false);
          e = -1;
        }
      }
      if (e == -1 && direct && bounce_usable.load()) {
        uint8_t *b = bounce.fit(j.len);
        if (b) {
          e = read_all(fd_direct, b, j.len, j.off);
          if (e == 0) std::memcpy(j.ptr, b, j.len);
          if (e == EINVAL) {
            bounce_usable.store(false);
            e = -1;
          }
        }
      }
      if (e == -1) e = read_all(fd_buffered, (uint8_t *)j.ptr, j.len, j.off);
      {
        std::lock_guard<std::mutex> lk(sh.mu);
        if (e) sh.done[j.slot] = -e;  // the first failed piece decides; the slot is never submitted then
        if (--sh.left[j.slot] == 0 && sh.done[j.slot] == 0) sh.done[j.slot] = 1;
      }
      sh.cv.notify_all();
    }
  };
  int err_no = 0;
  try {
    for (uint32_t i = 0; i < threads; ++i) readers.emplace_back(reader);
  } catch (...) {
    rc = DS_ENOMEM;
  }
  uint64_t handed = 0, submitted = 0;
  bool eof = false;
  while (rc == DS_OK && (!eof || submitted < handed)) {
    // fill the window
    while (!eof && handed - submitted < window) {
      void *p = nullptr;
      uint64_t off = 0, len = 0;
      int r = ds_restore_next_slot(ev, &p, &off, &len);
      if (r == DS_EOF) { eof = true; break; }
      if (r == DS_EBUSY) break;  // the ring is smaller than the window: submit first
      if (r != DS_OK) { rc = r; break; }
      const int slot = (int)(handed % window);
      win[slot] = p;
      int pieces = 0;
      for_each_piece(targets, off, len, [&](uint32_t, uint64_t, uint64_t, uint64_t) { ++pieces; });
      {
        std::lock_guard<std::mutex> lk(sh.mu);
        sh.done[slot] = pieces ? 0 : 1;
        sh.left[slot] = pieces;
        for_each_piece(targets, off, len, [&](uint32_t t, uint64_t file_off, uint64_t in_slot, uint64_t n) {
          IoJob j;
          j.ptr = (uint8_t *)p + in_slot;
          j.off = file_off;
          j.len = n;
          j.slot = slot;
          j.target = t;
          sh.todo.push_back(j);
        });
      }
      sh.cv.notify_all();
      ++handed;
    }
    if (rc != DS_OK || submitted == handed) continue;
    // submit the oldest one once it has been read
    const int pos = (int)(submitted % window);
    int state;
    {
      std::unique_lock<std::mutex> lk(sh.mu);
      sh.cv.wait(lk, [&] { return sh.left[pos] == 0 && sh.done[pos] != 0; });
      state = sh.done[pos];
    }
    if (state < 0) {
      rc = DS_EIO;
      err_no = -state;
      break;
    }
    rc = ds_restore_submit(ev, win[pos]);
    ++submitted;
  }
  {
    std::lock_guard<std::mutex> lk(sh.mu);
    sh.stop = true;
    if (rc != DS_OK) sh.todo.clear();
  }
  sh.cv.notify_all();
  for (std::thread &t : readers)
    if (t.joinable()) t.join();
  if (rc != DS_OK) {
    g_last_errno = err_no;
    (void)ds_event_destroy(ev);
    return rc;
  }
  *out = ev;
  return DS_OK;
}

void ds_set_errno(int e) { g_last_errno = e; }

bool ds_io_uring_available() {
  Uring r;
  const bool ok = r.open_ring(4) == 0;
  r.close_ring();
  return ok;
}

extern "C" {

int ds_last_errno(void) { return g_last_errno; }

int ds_flush_start(ds_event *ev, const char *path, uint32_t threads, uint32_t flags, ds_flush **out) {
  if (!ev || !path || !out || (flags & ~(DS_FILE_DIRECT | DS_FILE_SYNC | DS_FILE_URING))) return DS_EINVAL;
  if (threads > 64) return DS_EINVAL;
  const int fd_buffered = open(path, O_WRONLY | O_CREAT | O_TRUNC | O_CLOEXEC, 0644);
  if (fd_buffered < 0) {
    g_last_errno = errno;
    return DS_EIO;
  }
  // direct I/O where the file system has it; chunks that are not 4 KiB-shaped take the buffered descriptor
  const int fd_direct = (flags & DS_FILE_DIRECT) ? open(path, O_WRONLY | O_DIRECT | O_CLOEXEC) : -1;
  int rc = ds_flush_start_fds(ev, fd_buffered, fd_direct, threads, flags, out);
  if (rc != DS_OK) {
    if (fd_direct >= 0) close(fd_direct);
    close(fd_buffered);
    return rc;
  }
  (*out)->own_fds = true;
  return DS_OK;
}

int ds_flush_start_files(ds_event *ev, const char *const *paths, uint32_t n_files, uint32_t threads, uint32_t flags,
                         ds_flush **out) {
  if (!ev || !paths || !out || (flags & ~(DS_FILE_DIRECT | DS_FILE_SYNC | DS_FILE_URING))) return DS_EINVAL;
  if (threads > 64) return DS_EINVAL;
  const ds_plan *plan = ds_event_plan(ev);
  if (!plan || (size_t)n_files + 1 != plan->file_begin.size()) return DS_EINVAL;
  for (uint32_t k = 0; k < n_files; ++k)
    if (!paths[k]) return DS_EINVAL;
  std::vector<DsFileTarget> targets;
  int rc = DS_OK;
  try {
    targets.resize(n_files);
  } catch (const std::bad_alloc &) {
    return DS_ENOMEM;
  }
  for (uint32_t k = 0; k < n_files && rc == DS_OK; ++k) {
    DsFileTarget &t = targets[k];
    t.begin = plan->file_begin[k];
    t.end = plan->file_begin[k + 1];
    t.fd_buffered = open(paths[k], O_WRONLY | O_CREAT | O_TRUNC | O_CLOEXEC, 0644);
    if (t.fd_buffered < 0) {
      g_last_errno = errno;
      rc = DS_EIO;
      break;
    }
    t.fd_direct = (flags & DS_FILE_DIRECT) ? open(paths[k], O_WRONLY | O_DIRECT | O_CLOEXEC) : -1;
  }
  if (rc == DS_OK) {
    try {
      rc = ds_flush_start_targets(ev, targets, threads, flags, out);
    } catch (const std::bad_alloc &) {
      rc = DS_ENOMEM;
    }
  }
  if (rc != DS_OK) {
    for (const DsFileTarget &t : targets) {
      if (t.fd_direct >= 0) close(t.fd_direct);
      if (t.fd_buffered >= 0) close(t.fd_buffered);
    }
    return rc;
  }
  (*out)->own_fds = true;
  return DS_OK;
}

int ds_flush_wait(ds_flush *f, uint64_t *bytes_written, double *seconds) {
  if (!f) return DS_EINVAL;
  if (f->dispatcher.joinable()) f->dispatcher.join();
  f->cv.notify_all();
  for (std::thread &t : f->writers)
    if (t.joinable()) t.join();
  int status = f->status.load();
  if (f->own_fds) {
    for (const DsFileTarget &t : f->targets) {
      if (status == DS_OK && (f->flags & DS_FILE_SYNC) && fsync(t.fd_buffered) != 0) {
        status = DS_EIO;
        f->err_no.store(errno);
      }
      if (t.fd_direct >= 0) close(t.fd_direct);
      if (close(t.fd_buffered) != 0 && status == DS_OK) {
        status = DS_EIO;
        f->err_no.store(errno);
      }
    }
  }
  f->t1 = now_s();
  if (bytes_written) *bytes_written = f->bytes.load();
  if (seconds) *seconds = f->t1 - f->t0;
  g_last_errno = f->err_no.load();
  delete f;
  return status;
}

int ds_restore_from_file(ds_engine *engine, const ds_plan *plan, const char *path, uint32_t threads, uint32_t flags,
                         void *compute_stream, ds_event **out) {
  if (!engine || !plan || !path || !out || (flags & ~DS_FILE_DIRECT)) return DS_EINVAL;
  if (threads > 64) return DS_EINVAL;
  DsFileTarget t;
  t.begin = 0;
  t.end = ~(uint64_t)0;
  t.fd_buffered = open(path, O_RDONLY | O_CLOEXEC);
  if (t.fd_buffered < 0) {
    g_last_errno = errno;
    return DS_EIO;
  }
  t.fd_direct = (flags & DS_FILE_DIRECT) ? open(path, O_RDONLY | O_DIRECT | O_CLOEXEC) : -1;
  int rc;
  try {
    rc = ds_restore_from_targets(engine, plan, std::vector<DsFileTarget>(1, t), threads, compute_stream, out);
  } catch (const std::bad_alloc &) {
    rc = DS_ENOMEM;
  }
  if (t.fd_direct >= 0) close(t.fd_direct);
  close(t.fd_buffered);
  return rc;
}

int ds_restore_from_files(ds_engine *engine, const ds_plan *plan, const char *const *paths, uint32_t n_files,
                          uint32_t threads, uint32_t flags, void *compute_stream, ds_event **out) {
  if (!engine || !plan || !paths || !out || (flags & ~DS_FILE_DIRECT)) return DS_EINVAL;
  if (threads > 64 || (size_t)n_files + 1 != plan->file_begin.size()) return DS_EINVAL;
  for (uint32_t k = 0; k < n_files; ++k)
    if (!paths[k]) return DS_EINVAL;
  std::vector<DsFileTarget> targets;
  int rc = DS_OK;
  try {
    targets.resize(n_files);
  } catch (const std::bad_alloc &) {
    return DS_ENOMEM;
  }
  for (uint32_t k = 0; k < n_files; ++k) {
    DsFileTarget &t = targets[k];
    t.begin = plan->file_begin[k];
    t.end = plan->file_begin[k + 1];
    t.fd_buffered = open(paths[k], O_RDONLY | O_CLOEXEC);
    if (t.fd_buffered < 0) {
      g_last_errno = errno;
      rc = DS_EIO;
      break;
    }
    t.fd_direct = (flags & DS_FILE_DIRECT) ? open(paths[k], O_RDONLY | O_DIRECT | O_CLOEXEC) : -1;
  }
  if (rc == DS_OK) {
    try {
      rc = ds_restore_from_targets(engine, plan, targets, threads, compute_stream, out);
    } catch (const std::bad_alloc &) {
      rc = DS_ENOMEM;
    }
  }
  const int keep = g_last_errno;
  for (const DsFileTarget &t : targets) {
    if (t.fd_direct >= 0) close(t.fd_direct);
    if (t.fd_buffered >= 0) close(t.fd_buffered);
  }
  g_last_errno = keep;
  return rc;
}

}  // extern "C"
