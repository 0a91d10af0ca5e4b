// The checkpoint file (DataStates-LLM Sec. V-A5): (1) tensors at offsets known
// in advance -- the plan's image is the head of the file; (2) serialized
// objects, whose sizes are not known in advance, appended behind the tensors
// as a concurrent log while the tensors are still being flushed; (3) a
// metadata header written last, at the end of the file, from which both kinds
// can be recovered.  The byte encoding is documented in datastates.h.
#include <fcntl.h>
#include <sys/stat.h>
#include <unistd.h>

#include <algorithm>
#include <atomic>
#include <cerrno>
#include <chrono>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "ds_internal.h"

namespace {

constexpr char kMagic[8] = {'D', 'S', 'C', 'K', 'P', 'T', '0', '1'};
constexpr uint32_t kVersion = 1;
constexpr uint64_t kTensorEntry = 80, kChunkEntry = 32, kFooter = 64;

struct ChunkEntry {
  uint64_t object_id, seq, off, len;
};

// CRC-32 of IEEE 802.3 (reflected polynomial 0xEDB88320, initial value and final xor 0xFFFFFFFF)
uint32_t crc32_ieee(const uint8_t *p, size_t n, uint32_t crc = 0) {
  static uint32_t table[256];
  static std::once_flag once;
  std::call_once(once, [] {
    for (uint32_t i = 0; i < 256; ++i) {
      uint32_t c = i;
      for (int k = 0; k < 8; ++k) c = (c & 1) ? 0xEDB88320u ^ (c >> 1) : c >> 1;
      table[i] = c;
    }
  });
  crc = ~crc;
  for (size_t i = 0; i < n; ++i) crc = table[(crc ^ p[i]) & 0xFF] ^ (crc >> 8);
  return ~crc;
}

void put32(std::vector<uint8_t> &b, uint32_t v) {
  for (int i = 0; i < 4; ++i) b.push_back((uint8_t)(v >> (8 * i)));
}
void put64(std::vector<uint8_t> &b, uint64_t v) {
  for (int i = 0; i < 8; ++i) b.push_back((uint8_t)(v >> (8 * i)));
}
uint32_t get32(const uint8_t *p) {
  uint32_t v = 0;
  for (int i = 0; i < 4; ++i) v |= (uint32_t)p[i] << (8 * i);
  return v;
}
uint64_t get64(const uint8_t *p) {
  uint64_t v = 0;
  for (int i = 0; i < 8; ++i) v |= (uint64_t)p[i] << (8 * i);
  return v;
}

int pwrite_all(int fd, const uint8_t *p, uint64_t len, uint64_t off) {
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
int pread_all(int fd, uint8_t *p, uint64_t len, uint64_t off) {
  while (len) {
    ssize_t r = pread(fd, p, len, (off_t)off);
    if (r < 0) {
      if (errno == EINTR) continue;
      return errno;
    }
    if (r == 0) return EIO;
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

// One flush that feeds the files of several writers: the first of them to finish waits for it, all of them
// get its status, the last one frees it.
struct SharedFlush {
  ds_flush *flush = nullptr;
  std::mutex mu;
  bool waited = false;
  int status = DS_OK, err_no = 0;
  int refs = 0;
};

struct ds_ckpt {
  const ds_plan *plan = nullptr;
  uint32_t file = 0;      // which of the plan's files this is
  uint64_t region = 0;    // length of its tensor region
  int fd = -1, fd_direct = -1;
  uint32_t flags = 0;
  ds_flush *flush = nullptr;
  SharedFlush *shared = nullptr;
  std::atomic<uint64_t> tail{0};  // next free byte of the log
  std::mutex mu;                  // chunks, next_seq, status
  std::vector<ChunkEntry> chunks;
  std::map<uint64_t, uint64_t> next_seq;
  int status = DS_OK, err_no = 0;
  double t0 = 0;
};

struct ds_ckpt_reader {
  std::string path;
  int fd = -1;
  ds_ckpt_layout lay{};
  std::vector<ds_ckpt_tensor> tensors;
  std::vector<ChunkEntry> chunks;            // sorted by (object_id, seq)
  std::vector<std::pair<uint64_t, uint64_t>> objects;  // (id, bytes), ascending id
  std::vector<size_t> first_chunk;           // per object: index of its chunk 0
};

extern "C" {

int ds_ckpt_create(const char *path, const ds_plan *plan, uint32_t flags, ds_ckpt **out) {
  if (!plan || plan->file_begin.size() != 2) return DS_EINVAL;  // a plan of several files: one writer per part
  return ds_ckpt_create_part(path, plan, 0, flags, out);
}

int ds_ckpt_create_part(const char *path, const ds_plan *plan, uint32_t file, uint32_t flags, ds_ckpt **out) {
  if (!path || !plan || !out || (flags & ~(DS_FILE_DIRECT | DS_FILE_SYNC | DS_FILE_URING))) return DS_EINVAL;
  if ((size_t)file + 1 >= plan->file_begin.size()) return DS_EINVAL;
  ds_ckpt *c = new (std::nothrow) ds_ckpt;
  if (!c) return DS_ENOMEM;
  c->fd = open(path, O_RDWR | O_CREAT | O_TRUNC | O_CLOEXEC, 0644);
  if (c->fd < 0) {
    ds_set_errno(errno);
    delete c;
    return DS_EIO;
  }
  if (flags & DS_FILE_DIRECT) c->fd_direct = open(path, O_WRONLY | O_DIRECT | O_CLOEXEC);
  c->plan = plan;
  c->file = file;
  c->region = plan->file_begin[file + 1] - plan->file_begin[file];
  c->flags = flags;
  c->tail.store(c->region);  // a multiple of the alignment (>= 16), so of 8
  c->t0 = now_s();
  *out = c;
  return DS_OK;
}

int ds_ckpt_flush_snapshot(ds_ckpt *c, ds_event *snapshot, uint32_t threads) {
  if (!c || !snapshot) return DS_EINVAL;
  if (c->flush || c->shared) return DS_ESTATE;
  if (c->plan->file_begin.size() != 2) return DS_EINVAL;  // parts are flushed together
  return ds_flush_start_fds(snapshot, c->fd, c->fd_direct, threads, c->flags & (DS_FILE_DIRECT | DS_FILE_URING),
                            &c->flush);
}

int ds_ckpt_flush_snapshot_parts(ds_ckpt *const *parts, uint32_t n_parts, ds_event *snapshot, uint32_t threads) {
  if (!parts || !n_parts || !snapshot) return DS_EINVAL;
  const ds_plan *plan = ds_event_plan(snapshot);
  if (!plan || (size_t)n_parts + 1 != plan->file_begin.size()) return DS_EINVAL;
  for (uint32_t k = 0; k < n_parts; ++k) {
    if (!parts[k] || parts[k]->plan != plan || parts[k]->file != k) return DS_EINVAL;
    if (parts[k]->flush || parts[k]->shared) return DS_ESTATE;
  }
  SharedFlush *sf = new (std::nothrow) SharedFlush;
  if (!sf) return DS_ENOMEM;
  int rc;
  try {
    std::vector<DsFileTarget> targets(n_parts);
    for (uint32_t k = 0; k < n_parts; ++k) {
      targets[k].begin = plan->file_begin[k];
      targets[k].end = plan->file_begin[k + 1];
      targets[k].fd_buffered = parts[k]->fd;
      targets[k].fd_direct = parts[k]->fd_direct;
    }
    rc = ds_flush_start_targets(snapshot, std::move(targets), threads,
                                parts[0]->flags & (DS_FILE_DIRECT | DS_FILE_URING), &sf->flush);
  } catch (const std::bad_alloc &) {
    rc = DS_ENOMEM;
  }
  if (rc != DS_OK) {
    delete sf;
    return rc;
  }
  sf->refs = (int)n_parts;
  for (uint32_t k = 0; k < n_parts; ++k) parts[k]->shared = sf;
  return DS_OK;
}

int ds_ckpt_write_region(ds_ckpt *c, uint64_t file_off, const void *host, uint64_t len) {
  if (!c || (!host && len)) return DS_EINVAL;
  if (file_off > c->region || len > c->region - file_off) return DS_ERANGE;
  const int e = pwrite_all(c->fd, (const uint8_t *)host, len, file_off);
  if (e) {
    ds_set_errno(e);
    return DS_EIO;
  }
  return DS_OK;
}

int ds_ckpt_append(ds_ckpt *c, uint64_t object_id, const void *data, uint64_t len) {
  if (!c || (!data && len) || len > ((uint64_t)1 << 60)) return DS_EINVAL;
  ChunkEntry ce;
  ce.object_id = object_id;
  ce.len = len;
  ce.off = c->tail.fetch_add((len + 7) & ~(uint64_t)7);  // the claim: nobody else writes there
  {
    std::lock_guard<std::mutex> lk(c->mu);
    ce.seq = c->next_seq[object_id]++;
    c->chunks.push_back(ce);
  }
  const int e = pwrite_all(c->fd, (const uint8_t *)data, len, ce.off);
  if (e) {
    std::lock_guard<std::mutex> lk(c->mu);
    if (c->status == DS_OK) {
      c->status = DS_EIO;
      c->err_no = e;
    }
    ds_set_errno(e);
    return DS_EIO;
  }
  return DS_OK;
}

int ds_ckpt_append_from(ds_ckpt *c, uint64_t object_id, ds_chunk_provider next, void *ctx, uint64_t *n_chunks) {
  if (!c || !next) return DS_EINVAL;
  uint64_t count = 0;
  int rc = DS_OK;
  for (;;) {
    const void *data = nullptr;
    uint64_t len = 0;
    const int more = next(ctx, &data, &len);
    if (more < 0) { rc = more; break; }   // the provider's own error, handed through
    if (more == 0) break;
    rc = ds_ckpt_append(c, object_id, data, len);
    if (rc != DS_OK) break;
    ++count;
  }
  if (n_chunks) *n_chunks = count;
  return rc;
}

int ds_ckpt_finish(ds_ckpt *c, uint64_t *file_bytes, double *seconds) {
  if (!c) return DS_EINVAL;
  int status = DS_OK, err_no = 0;
  if (c->flush) {
    status = ds_flush_wait(c->flush, nullptr, nullptr);
    if (status != DS_OK) err_no = ds_last_errno();
    c->flush = nullptr;
  }
  if (c->shared) {
    SharedFlush *sf = c->shared;
    bool last;
    {
      std::lock_guard<std::mutex> lk(sf->mu);
      if (!sf->waited) {
        sf->status = ds_flush_wait(sf->flush, nullptr, nullptr);
        sf->err_no = sf->status != DS_OK ? ds_last_errno() : 0;
        sf->flush = nullptr;
        sf->waited = true;
      }
      status = sf->status;
      err_no = sf->err_no;
      last = --sf->refs == 0;
    }
    if (last) delete sf;
    c->shared = nullptr;
  }
  if (status == DS_OK && c->status != DS_OK) {
    status = c->status;
    err_no = c->err_no;
  }
  uint64_t end = 0;
  if (status == DS_OK) {
    const ds_plan *p = c->plan;
    std::sort(c->chunks.begin(), c->chunks.end(), [](const ChunkEntry &a, const ChunkEntry &b) {
      return a.object_id != b.object_id ? a.object_id < b.object_id : a.seq < b.seq;
    });
    std::vector<uint8_t> t;
    try {
      uint64_t n_mine = 0;
      for (const DsManifestEntry &m : p->manifest) n_mine += m.file == c->file;
      t.reserve(n_mine * kTensorEntry + c->chunks.size() * kChunkEntry + kFooter);
      for (const DsManifestEntry &m : p->manifest) {
        if (m.file != c->file) continue;
        put64(t, m.tensor_id);
        put32(t, m.dtype);
        put32(t, m.ndim);
        for (int j = 0; j < DS_MAX_DIMS; ++j) put64(t, (uint64_t)m.shape[j]);
        put64(t, m.file_offset);
        put64(t, m.nbytes);
      }
      for (const ChunkEntry &ce : c->chunks) {
        put64(t, ce.object_id);
        put64(t, ce.seq);
        put64(t, ce.off);
        put64(t, ce.len);
      }
      const uint32_t trailer_crc = crc32_ieee(t.data(), t.size());
      const size_t f0 = t.size();
      for (char ch : kMagic) t.push_back((uint8_t)ch);
      put32(t, kVersion);
      put32(t, 0);
      put64(t, p->align);
      put64(t, c->region);
      put64(t, c->tail.load());
      put64(t, n_mine);
      put64(t, c->chunks.size());
      put32(t, trailer_crc);
      put32(t, crc32_ieee(t.data() + f0, 60));
    } catch (const std::bad_alloc &) {
      status = DS_ENOMEM;
    }
    if (status == DS_OK) {
      const int e = pwrite_all(c->fd, t.data(), t.size(), c->tail.load());
      if (e) {
        status = DS_EIO;
        err_no = e;
      }
      end = c->tail.load() + t.size();
    }
    if (status == DS_OK && (c->flags & DS_FILE_SYNC) && fsync(c->fd) != 0) {
      status = DS_EIO;
      err_no = errno;
    }
  }
  if (c->fd_direct >= 0) close(c->fd_direct);
  if (close(c->fd) != 0 && status == DS_OK) {
    status = DS_EIO;
    err_no = errno;
  }
  if (file_bytes) *file_bytes = end;
  if (seconds) *seconds = now_s() - c->t0;
  if (status == DS_EIO) ds_set_errno(err_no);
  delete c;
  return status;
}

int ds_ckpt_open(const char *path, ds_ckpt_reader **out) {
  if (!path || !out) return DS_EINVAL;
  ds_ckpt_reader *r = new (std::nothrow) ds_ckpt_reader;
  if (!r) return DS_ENOMEM;
  int rc = DS_OK;
  try {
    r->path = path;
    r->fd = open(path, O_RDONLY | O_CLOEXEC);
    struct stat st;
    if (r->fd < 0 || fstat(r->fd, &st) != 0) {
      ds_set_errno(errno);
      rc = DS_EIO;
    }
    uint8_t f[kFooter];
    uint64_t size = 0, n = 0, m = 0, T = 0, E = 0, align = 0;
    if (rc == DS_OK) {
      size = (uint64_t)st.st_size;
      if (size < kFooter) rc = DS_EFORMAT;
    }
    if (rc == DS_OK) {
      const int e = pread_all(r->fd, f, kFooter, size - kFooter);
      if (e) {
        ds_set_errno(e);
        rc = DS_EIO;
      }
    }
    if (rc == DS_OK) {
      if (std::memcmp(f, kMagic, 8) != 0 || get32(f + 8) != kVersion || get32(f + 12) != 0 ||
          get32(f + 60) != crc32_ieee(f, 60))
        rc = DS_EFORMAT;
    }
    if (rc == DS_OK) {
      align = get64(f + 16);
      T = get64(f + 24);
      E = get64(f + 32);
      n = get64(f + 40);
      m = get64(f + 48);
      // sizes first, so that nothing below can overflow
      const uint64_t lim = size / kChunkEntry + 1;
      if (n > lim || m > lim || E > size || T > E || (E & 7) || align < 16 || (align & (align - 1)) ||
          (T & (align - 1)) || E + n * kTensorEntry + m * kChunkEntry + kFooter != size)
        rc = DS_EFORMAT;
    }
    std::vector<uint8_t> t;
    if (rc == DS_OK) {
      t.resize(n * kTensorEntry + m * kChunkEntry);
      const int e = t.empty() ? 0 : pread_all(r->fd, t.data(), t.size(), E);
      if (e) {
        ds_set_errno(e);
        rc = DS_EIO;
      } else if (crc32_ieee(t.data(), t.size()) != get32(f + 56)) {
        rc = DS_EFORMAT;
      }
    }
    if (rc == DS_OK) {
      r->tensors.resize(n);
      for (uint64_t i = 0; i < n && rc == DS_OK; ++i) {
        const uint8_t *q = t.data() + i * kTensorEntry;
        ds_ckpt_tensor &x = r->tensors[i];
        x.tensor_id = get64(q);
        x.dtype = get32(q + 8);
        x.ndim = get32(q + 12);
        for (int j = 0; j < DS_MAX_DIMS; ++j) x.shape[j] = (int64_t)get64(q + 16 + 8 * j);
        x.file_offset = get64(q + 64);
        x.nbytes = get64(q + 72);
        if (x.ndim > DS_MAX_DIMS || ds_itemsize(x.dtype) == 0 || (x.file_offset & (align - 1)) ||
            x.file_offset > T || x.nbytes > T - x.file_offset)
          rc = DS_EFORMAT;
      }
      r->chunks.resize(m);
      for (uint64_t k = 0; k < m && rc == DS_OK; ++k) {
        const uint8_t *q = t.data() + n * kTensorEntry + k * kChunkEntry;
        ChunkEntry &ce = r->chunks[k];
        ce.object_id = get64(q);
        ce.seq = get64(q + 8);
        ce.off = get64(q + 16);
        ce.len = get64(q + 24);
        if (ce.off < T || ce.off > E || ce.len > E - ce.off) rc = DS_EFORMAT;
        const bool first = k == 0 || r->chunks[k - 1].object_id != ce.object_id;
        if (first) {
          if (ce.seq != 0 || (k && r->chunks[k - 1].object_id > ce.object_id)) rc = DS_EFORMAT;
          r->objects.emplace_back(ce.object_id, 0);
          r->first_chunk.push_back(k);
        } else if (ce.seq != r->chunks[k - 1].seq + 1) {
          rc = DS_EFORMAT;
        }
        if (rc == DS_OK) r->objects.back().second += ce.len;
      }
    }
    if (rc == DS_OK) {
      r->lay.align = align;
      r->lay.tensor_bytes = T;
      r->lay.log_end = E;
      r->lay.n_tensors = n;
      r->lay.n_chunks = m;
      r->lay.n_objects = r->objects.size();
      r->lay.file_bytes = size;
    }
  } catch (const std::bad_alloc &) {
    rc = DS_ENOMEM;
  }
  if (rc != DS_OK) {
    if (r->fd >= 0) close(r->fd);
    delete r;
    return rc;
  }
  *out = r;
  return DS_OK;
}

int ds_ckpt_close(ds_ckpt_reader *r) {
  if (!r) return DS_EINVAL;
  close(r->fd);
  delete r;
  return DS_OK;
}

int ds_ckpt_layout_info(const ds_ckpt_reader *r, ds_ckpt_layout *out) {
  if (!r || !out) return DS_EINVAL;
  *out = r->lay;
  return DS_OK;
}

int ds_ckpt_tensor_info(const ds_ckpt_reader *r, size_t i, ds_ckpt_tensor *out) {
  if (!r || !out || i >= r->tensors.size()) return DS_EINVAL;
  *out = r->tensors[i];
  return DS_OK;
}

int ds_ckpt_object_at(const ds_ckpt_reader *r, size_t k, uint64_t *object_id, uint64_t *nbytes) {
  if (!r || k >= r->objects.size()) return DS_EINVAL;
  if (object_id) *object_id = r->objects[k].first;
  if (nbytes) *nbytes = r->objects[k].second;
  return DS_OK;
}

int ds_ckpt_object_read(const ds_ckpt_reader *r, uint64_t object_id, void *buf, uint64_t cap, uint64_t *len) {
  if (!r) return DS_EINVAL;
  auto it = std::lower_bound(r->objects.begin(), r->objects.end(), std::make_pair(object_id, (uint64_t)0));
  if (it == r->objects.end() || it->first != object_id) return DS_EINVAL;
  if (len) *len = it->second;
  if (it->second > cap) return DS_ERANGE;
  if (it->second && !buf) return DS_EINVAL;
  uint8_t *p = (uint8_t *)buf;
  for (size_t k = r->first_chunk[it - r->objects.begin()]; k < r->chunks.size() && r->chunks[k].object_id == object_id; ++k) {
    const int e = pread_all(r->fd, p, r->chunks[k].len, r->chunks[k].off);
    if (e) {
      ds_set_errno(e);
      return DS_EIO;
    }
    p += r->chunks[k].len;
  }
  return DS_OK;
}

int ds_ckpt_matches_plan(const ds_ckpt_reader *r, const ds_plan *plan) {
  if (!r || !plan) return DS_EINVAL;
  if (plan->file_begin.size() != 2) return DS_EINVAL;
  return ds_ckpt_matches_plan_part(r, plan, 0);
}

int ds_ckpt_matches_plan_part(const ds_ckpt_reader *r, const ds_plan *plan, uint32_t file) {
  if (!r || !plan || (size_t)file + 1 >= plan->file_begin.size()) return DS_EINVAL;
  if (r->lay.align != plan->align || r->lay.tensor_bytes != plan->file_begin[file + 1] - plan->file_begin[file])
    return DS_EFORMAT;
  size_t k = 0;  // the file's entries are the plan's entries of that file, in table order
  for (const DsManifestEntry &m : plan->manifest) {
    if (m.file != file) continue;
    if (k >= r->tensors.size()) return DS_EFORMAT;
    const ds_ckpt_tensor &x = r->tensors[k++];
    if (x.tensor_id != m.tensor_id || x.dtype != m.dtype || x.ndim != m.ndim || x.file_offset != m.file_offset ||
        x.nbytes != m.nbytes || std::memcmp(x.shape, m.shape, sizeof(x.shape)) != 0)
      return DS_EFORMAT;
  }
  return k == r->tensors.size() ? DS_OK : DS_EFORMAT;
}

int ds_ckpt_restore(const ds_ckpt_reader *r, ds_engine *engine, const ds_plan *plan, uint32_t threads, uint32_t flags,
                    void *compute_stream, ds_event **out) {
  if (!r || !engine || !plan || !out) return DS_EINVAL;
  const int rc = ds_ckpt_matches_plan(r, plan);
  if (rc != DS_OK) return rc;
  return ds_restore_from_file(engine, plan, r->path.c_str(), threads, flags, compute_stream, out);
}

int ds_ckpt_restore_parts(const ds_ckpt_reader *const *readers, uint32_t n_parts, ds_engine *engine,
                          const ds_plan *plan, uint32_t threads, uint32_t flags, void *compute_stream,
                          ds_event **out) {
  if (!readers || !engine || !plan || !out || (flags & ~DS_FILE_DIRECT)) return DS_EINVAL;
  if ((size_t)n_parts + 1 != plan->file_begin.size()) return DS_EINVAL;
  for (uint32_t k = 0; k < n_parts; ++k) {
    if (!readers[k]) return DS_EINVAL;
    const int rc = ds_ckpt_matches_plan_part(readers[k], plan, k);
    if (rc != DS_OK) return rc;
  }
  int rc;
  std::vector<DsFileTarget> targets;
  try {
    targets.resize(n_parts);
    for (uint32_t k = 0; k < n_parts; ++k) {
      targets[k].begin = plan->file_begin[k];
      targets[k].end = plan->file_begin[k + 1];
      targets[k].fd_buffered = readers[k]->fd;  // stays the reader's
      targets[k].fd_direct =
          (flags & DS_FILE_DIRECT) ? open(readers[k]->path.c_str(), O_RDONLY | O_DIRECT | O_CLOEXEC) : -1;
    }
    rc = ds_restore_from_targets(engine, plan, targets, threads, compute_stream, out);
  } catch (const std::bad_alloc &) {
    rc = DS_ENOMEM;
  }
  const int keep = ds_last_errno();
  for (const DsFileTarget &t : targets)
    if (t.fd_direct >= 0) close(t.fd_direct);
  ds_set_errno(keep);
  return rc;
}

}  // extern "C"
