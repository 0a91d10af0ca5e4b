// Host side of the plan: validation of the shard table, the image layout
// (DataStates-LLM Sec. V-A3 duty (a): sizes and offsets in the stream; Sec.
// V-A5 rule (1): tensor offsets are fixed in advance from the sizes), the
// normalisation of views and the work-group chunk table.
#include <algorithm>
#include <atomic>
#include <cstring>
#include <new>
#include <numeric>

#include "ds_internal.h"

namespace {

thread_local int g_last_hip_error = 0;

std::atomic<uint64_t> g_chunk_bytes{16u << 10};
std::atomic<uint64_t> g_variant{0};
std::atomic<uint64_t> g_grid_limit{0};

inline bool is_pow2(uint64_t x) { return x && !(x & (x - 1)); }
inline uint64_t round_up(uint64_t x, uint64_t a) { return (x + a - 1) & ~(a - 1); }

// bytes of a shard; false if the descriptor is malformed or the size overflows
bool shard_bytes(const ds_shard_desc &d, uint64_t *bytes) {
  int es = ds_itemsize(d.dtype);
  if (es == 0 || d.ndim > DS_MAX_DIMS) return false;
  unsigned __int128 n = 1;
  for (uint32_t j = 0; j < d.ndim; ++j) {
    if (d.shape[j] < 0) return false;
    n *= (unsigned __int128)(uint64_t)d.shape[j];
    if (n > ((unsigned __int128)1 << 62)) {
      // keep multiplying only if a later extent is zero (then the shard is empty)
      bool later_zero = false;
      for (uint32_t k = j + 1; k < d.ndim; ++k) later_zero |= (d.shape[k] == 0);
      if (!later_zero) return false;
      n = 0;
      break;
    }
  }
  n *= (unsigned)es;
  if (n > ((unsigned __int128)1 << 62)) return false;
  *bytes = (uint64_t)n;
  return true;
}

// A view must not address an element twice, else the scatter is ill-defined.
// Quick test, sufficient but not necessary: order the dimensions with extent > 1 by stride; every
// stride exceeds the largest displacement reachable with all smaller ones (true of every slice,
// transpose and permutation of a dense parent).  A view that fails it can still be injective --
// shape (3,2) with strides (2,3) addresses 0,3,2,5,4,7 -- so up to kEnumerateLimit elements the
// displacements are then written out and compared; larger views of that kind are refused.
constexpr uint64_t kEnumerateLimit = (uint64_t)1 << 20;

bool view_is_injective(const ds_shard_desc &d) {
  struct Dim { uint64_t extent, stride; };
  Dim dims[DS_MAX_DIMS];
  int m = 0;
  for (uint32_t j = 0; j < d.ndim; ++j) {
    if (d.shape[j] > 1) {
      if (d.strides[j] <= 0) return false;
      dims[m++] = {(uint64_t)d.shape[j], (uint64_t)d.strides[j]};
    }
  }
  std::sort(dims, dims + m, [](const Dim &a, const Dim &b) { return a.stride < b.stride; });
  unsigned __int128 reach = 0;  // largest displacement of the dimensions seen so far
  bool nested = true;
  for (int k = 0; k < m; ++k) {
    if ((unsigned __int128)dims[k].stride <= reach) nested = false;
    reach += (unsigned __int128)(dims[k].extent - 1) * dims[k].stride;
    if (reach > ((unsigned __int128)1 << 62)) return false;
  }
  if (nested) return true;
  uint64_t count = 1;
  for (int k = 0; k < m; ++k) {
    if (dims[k].extent > kEnumerateLimit / count) return false;  // too large to write out
    count *= dims[k].extent;
  }
  std::vector<uint64_t> at(1, 0);
  at.reserve(count);
  for (int k = 0; k < m; ++k) {
    const size_t have = at.size();
    for (uint64_t i = 1; i < dims[k].extent; ++i)
      for (size_t j = 0; j < have; ++j) at.push_back(at[j] + i * dims[k].stride);
  }
  std::sort(at.begin(), at.end());
  return std::adjacent_find(at.begin(), at.end()) == at.end();
}

// DS_PLAN_CHECK_MEMORY: every address of a non-empty view, from its base to its last element's last byte,
// must lie in the allocation the runtime reports for the base address.
int view_in_one_allocation(const ds_shard_desc &d) {
  unsigned __int128 last = 0;  // element index of the view's last element
  for (uint32_t j = 0; j < d.ndim; ++j) last += (unsigned __int128)(uint64_t)(d.shape[j] - 1) * (uint64_t)d.strides[j];
  const unsigned __int128 span = (last + 1) * (unsigned)ds_itemsize(d.dtype);
  hipDeviceptr_t abase = nullptr;
  size_t asize = 0;
  if (hipMemGetAddressRange(&abase, &asize, (hipDeviceptr_t)d.base) != hipSuccess) {
    (void)hipGetLastError();  // not memory the runtime knows: the error is reported through the return code
    return DS_EFAULT;
  }
  const uintptr_t b = (uintptr_t)d.base, a = (uintptr_t)abase;
  if (b < a || span > (unsigned __int128)asize || (unsigned __int128)(b - a) > (unsigned __int128)asize - span)
    return DS_EFAULT;
  return DS_OK;
}

// Device form of one non-empty shard: drop extents of 1, merge neighbouring
// dimensions that are contiguous with each other (stride[j] == extent[j+1] *
// stride[j+1]; this keeps the row-major order of the view), then split off the
// innermost run if its stride is one element.
DsTile make_tile(const ds_shard_desc &d, uint64_t nbytes) {
  const uint64_t es = (uint64_t)ds_itemsize(d.dtype);
  uint64_t ext[DS_MAX_DIMS], str[DS_MAX_DIMS];
  int m = 0;
  for (uint32_t j = 0; j < d.ndim; ++j) {
    if (d.shape[j] == 1) continue;
    uint64_t e = (uint64_t)d.shape[j], s = (uint64_t)d.strides[j];
    if (m > 0 && str[m - 1] == e * s) {
      ext[m - 1] *= e;
      str[m - 1] = s;
    } else {
      ext[m] = e;
      str[m] = s;
      ++m;
    }
  }
  DsTile t;
  std::memset(&t, 0, sizeof(t));
  t.src = (uint64_t)(uintptr_t)d.base;
  t.nbytes = nbytes;
  t.es_log2 = es == 8 ? 3 : es == 4 ? 2 : es == 2 ? 1 : 0;
  if (m > 0 && str[m - 1] == 1) {
    t.run_bytes = ext[m - 1] * es;
    --m;
  } else {
    t.run_bytes = es;
  }
  t.n_outer = (uint32_t)m;
  for (int j = 0; j < m; ++j) {
    t.extent[j] = ext[j];
    t.stride[j] = str[j] * es;
  }
  if (m == 0) t.run_bytes = nbytes;
  return t;
}

int upload(ds_plan *p) {
  DS_HIP_TRY(hipGetDevice(&p->device));
  const size_t b_tiles = p->tiles.size() * sizeof(DsTile);
  const size_t b_hot = round_up(p->hot.size() * sizeof(DsTileHot), 128);
  const size_t b_first = round_up(p->first_tile.size() * sizeof(uint32_t), 128);
  const size_t b_recs = round_up(p->recs.size() * sizeof(DsChunkRec), 128);
  const size_t total = std::max<size_t>(b_tiles + b_hot + b_first + b_recs, 128);
  DS_HIP_TRY(hipMalloc(&p->dev_blob, total));
  uint8_t *base = (uint8_t *)p->dev_blob;
  p->d_tiles = (const DsTile *)base;
  p->d_hot = (const DsTileHot *)(base + b_tiles);
  p->d_first_tile = (const uint32_t *)(base + b_tiles + b_hot);
  if (b_tiles) DS_HIP_TRY(hipMemcpy(base, p->tiles.data(), b_tiles, hipMemcpyHostToDevice));
  DS_HIP_TRY(hipMemcpy(base + b_tiles, p->hot.data(), p->hot.size() * sizeof(DsTileHot), hipMemcpyHostToDevice));
  DS_HIP_TRY(hipMemcpy(base + b_tiles + b_hot, p->first_tile.data(), p->first_tile.size() * sizeof(uint32_t),
                       hipMemcpyHostToDevice));
  p->d_recs = (const DsChunkRec *)(base + b_tiles + b_hot + b_first);
  if (!p->recs.empty())
    DS_HIP_TRY(hipMemcpy(base + b_tiles + b_hot + b_first, p->recs.data(), p->recs.size() * sizeof(DsChunkRec),
                         hipMemcpyHostToDevice));
  return DS_OK;
}

}  // namespace

void ds_set_hip_error(hipError_t e) { g_last_hip_error = (int)e; }
uint64_t ds_cfg_chunk_bytes() { return g_chunk_bytes.load(); }
uint64_t ds_cfg_variant() { return g_variant.load(); }

extern "C" {

int ds_last_hip_error(void) { return g_last_hip_error; }

int ds_itemsize(uint32_t dtype) {
  switch (dtype) {
    case DS_F32: return 4;
    case DS_BF16: return 2;
    case DS_F16: return 2;
    case DS_I64: return 8;
    case DS_U8: return 1;
    default: return 0;
  }
}

const char *ds_strerror(int code) {
  switch (code) {
    case DS_OK: return "ok";
    case DS_NOT_READY: return "snapshot still in flight";
    case DS_EOF: return "no more chunks";
    case DS_EINVAL: return "invalid argument (null pointer, dtype, ndim, shape, stride, alignment or base address)";
    case DS_EALIGN: return "a file offset is not a multiple of the alignment";
    case DS_EOVERLAP: return "shards overlap in the image, or a view addresses an element twice";
    case DS_EGAP: return "hole in the image that is not alignment padding";
    case DS_ERANGE: return "image range outside the image, reversed, or not a multiple of 16";
    case DS_ENOMEM: return "out of memory";
    case DS_EHIP: return "a HIP call failed (see ds_last_hip_error)";
    case DS_EBUSY: return "work still in flight";
    case DS_ESTATE: return "call not valid in this state";
    case DS_EIO: return "a file operation failed (see ds_last_errno)";
    case DS_EFORMAT: return "not a checkpoint file of this format, or a damaged one";
    case DS_EFAULT: return "a shard's addresses are not all inside one device allocation";
    case DS_ETOOBIG: return "the plan's tables do not fit the static table memory of ds_pack_noalloc";
    default: return "unknown datastates status";
  }
}

int ds_config_set(const char *key, uint64_t value) {
  if (!key) return DS_EINVAL;
  if (!std::strcmp(key, "chunk_bytes")) {
    if (value != (8u << 10) && value != (16u << 10) && value != (32u << 10)) return DS_EINVAL;
    g_chunk_bytes.store(value);
    return DS_OK;
  }
  if (!std::strcmp(key, "variant")) {
    if (value > 5) return DS_EINVAL;
    g_variant.store(value);
    return DS_OK;
  }
  if (!std::strcmp(key, "grid_limit")) {
    if (value > 0x7FFFFFFF) return DS_EINVAL;
    g_grid_limit.store(value);
    return DS_OK;
  }
  if (!std::strcmp(key, "drop_pinned_cache")) {
    if (value) ds_drop_pinned_cache();
    return DS_OK;
  }
  return DS_EINVAL;
}

int ds_config_get(const char *key, uint64_t *value) {
  if (!key || !value) return DS_EINVAL;
  if (!std::strcmp(key, "chunk_bytes")) { *value = g_chunk_bytes.load(); return DS_OK; }
  if (!std::strcmp(key, "variant")) { *value = g_variant.load(); return DS_OK; }
  if (!std::strcmp(key, "grid_limit")) { *value = g_grid_limit.load(); return DS_OK; }
  if (!std::strcmp(key, "io_uring_available")) { *value = ds_io_uring_available() ? 1 : 0; return DS_OK; }
  return DS_EINVAL;
}

int ds_layout_assign(ds_shard_desc *desc, size_t n, uint64_t align, uint64_t *total) {
  if ((!desc && n) || !total || !is_pow2(align) || align < 16) return DS_EINVAL;
  std::vector<uint64_t> sizes(n);
  for (size_t i = 0; i < n; ++i)
    if (!shard_bytes(desc[i], &sizes[i])) return DS_EINVAL;
  uint64_t at = 0;
  for (size_t i = 0; i < n; ++i) {
    desc[i].file_offset = at;
    at = round_up(at + sizes[i], align);
  }
  *total = at;
  return DS_OK;
}

int ds_layout_assign_files(ds_shard_desc *desc, const uint32_t *file_of, size_t n, uint32_t n_files, uint64_t align,
                           uint64_t *region_bytes, uint64_t *total) {
  if ((!desc && n) || (!file_of && n) || !total || !is_pow2(align) || align < 16) return DS_EINVAL;
  if (n_files == 0 || n_files > DS_MAX_FILES) return DS_EINVAL;
  std::vector<uint64_t> sizes(n), at(n_files, 0);
  for (size_t i = 0; i < n; ++i)
    if (!shard_bytes(desc[i], &sizes[i]) || file_of[i] >= n_files) return DS_EINVAL;
  for (size_t i = 0; i < n; ++i) {
    uint64_t &a = at[file_of[i]];
    desc[i].file_offset = a;
    a = round_up(a + sizes[i], align);
  }
  uint64_t sum = 0;
  for (uint32_t f = 0; f < n_files; ++f) {
    if (region_bytes) region_bytes[f] = at[f];
    sum += at[f];
  }
  *total = sum;
  return DS_OK;
}

int ds_plan_create(const ds_shard_desc *desc, size_t n, uint64_t align, uint32_t flags, ds_plan **out) {
  return ds_plan_create_files(desc, nullptr, n, 1, align, flags, out);
}

int ds_plan_create_files(const ds_shard_desc *given, const uint32_t *file_of, size_t n, uint32_t n_files,
                         uint64_t align, uint32_t flags, ds_plan **out) {
  if ((!given && n) || !out || !is_pow2(align) || align < 16) return DS_EINVAL;
  if (n_files == 0 || n_files > DS_MAX_FILES || (!file_of && n_files > 1 && n)) return DS_EINVAL;
  if (flags & ~(DS_PLAN_STRICT | DS_PLAN_HOST_ONLY | DS_PLAN_CHECK_MEMORY)) return DS_EINVAL;
  if ((flags & DS_PLAN_CHECK_MEMORY) && (flags & DS_PLAN_HOST_ONLY)) return DS_EINVAL;
  ds_plan *p = new (std::nothrow) ds_plan;
  if (!p) return DS_ENOMEM;
  int rc = DS_OK;
  try {
    p->align = align;
    p->n_shards = n;
    p->manifest.resize(n);
    std::vector<uint64_t> sizes(n);
    // Several files: every file's tensor region (its shards at the offsets given, which count from the
    // start of THAT file) goes into the one image behind the regions of the files before it.  From here
    // on `desc` holds offsets in the image; the manifest keeps both.
    std::vector<ds_shard_desc> in_image;
    const ds_shard_desc *desc = given;
    p->file_begin.assign((size_t)n_files + 1, 0);
    if (file_of) {
      std::vector<uint64_t> region(n_files, 0);
      for (size_t i = 0; i < n && rc == DS_OK; ++i) {
        if (!shard_bytes(given[i], &sizes[i]) || file_of[i] >= n_files) { rc = DS_EINVAL; break; }
        if (given[i].file_offset > ((uint64_t)1 << 62)) { rc = DS_EINVAL; break; }
        region[file_of[i]] = std::max(region[file_of[i]], round_up(given[i].file_offset + sizes[i], align));
      }
      for (uint32_t f = 0; f < n_files && rc == DS_OK; ++f) {
        p->file_begin[f + 1] = p->file_begin[f] + region[f];
        if (p->file_begin[f + 1] > ((uint64_t)1 << 62)) rc = DS_EINVAL;
      }
      if (rc == DS_OK) {
        in_image.assign(given, given + n);
        for (size_t i = 0; i < n; ++i) in_image[i].file_offset += p->file_begin[file_of[i]];
        desc = in_image.data();
      }
    }
    uint64_t end_max = 0;
    for (size_t i = 0; i < n && rc == DS_OK; ++i) {
      const ds_shard_desc &d = desc[i];
      if (!shard_bytes(d, &sizes[i])) { rc = DS_EINVAL; break; }
      if (given[i].file_offset & (align - 1)) { rc = DS_EALIGN; break; }
      if (d.file_offset > ((uint64_t)1 << 62)) { rc = DS_EINVAL; break; }
      if (sizes[i]) {
        const uint64_t es = (uint64_t)ds_itemsize(d.dtype);
        if (!d.base || ((uint64_t)(uintptr_t)d.base % es)) { rc = DS_EINVAL; break; }
        bool bad_stride = false;
        for (uint32_t j = 0; j < d.ndim; ++j) bad_stride |= (d.shape[j] > 1 && d.strides[j] <= 0);
        if (bad_stride) { rc = DS_EINVAL; break; }
        if (!view_is_injective(d)) { rc = DS_EOVERLAP; break; }
        if (flags & DS_PLAN_CHECK_MEMORY) {
          rc = view_in_one_allocation(d);
          if (rc != DS_OK) break;
        }
      }
      DsManifestEntry &me = p->manifest[i];
      me.tensor_id = d.tensor_id;
      me.dtype = d.dtype;
      me.ndim = d.ndim;
      for (uint32_t j = 0; j < DS_MAX_DIMS; ++j) me.shape[j] = j < d.ndim ? d.shape[j] : 0;
      me.file_offset = given[i].file_offset;
      me.image_offset = d.file_offset;
      me.file = file_of ? file_of[i] : 0;
      me.nbytes = sizes[i];
      p->payload_bytes += sizes[i];
      end_max = std::max(end_max, d.file_offset + sizes[i]);
    }
    if (rc == DS_OK) {
      // one file: up to the end of the last shard; several: the regions, which cover that
      if (file_of) p->total_bytes = p->file_begin[n_files];
      else p->total_bytes = p->file_begin[1] = round_up(end_max, align);
      // image order of the non-empty shards
      std::vector<size_t> order;
      order.reserve(n);
      for (size_t i = 0; i < n; ++i) if (sizes[i]) order.push_back(i);
      std::sort(order.begin(), order.end(),
                [&](size_t a, size_t b) { return desc[a].file_offset < desc[b].file_offset; });
      // overlaps first (over the whole table), holes second: the code returned for a table with
      // both kinds of mistake does not depend on where they are
      uint64_t prev_end = 0;  // end of the shard before, in the image
      for (size_t k = 0; k < order.size() && rc == DS_OK; ++k) {
        const ds_shard_desc &d = desc[order[k]];
        if (d.file_offset < prev_end) { rc = DS_EOVERLAP; break; }
        prev_end = d.file_offset + sizes[order[k]];
      }
      if (rc == DS_OK && (flags & DS_PLAN_STRICT)) {
        prev_end = 0;
        for (size_t k = 0; k < order.size(); ++k) {
          const ds_shard_desc &d = desc[order[k]];
          if (d.file_offset > round_up(prev_end, align)) { rc = DS_EGAP; break; }
          prev_end = d.file_offset + sizes[order[k]];
        }
        if (rc == DS_OK && p->total_bytes > round_up(prev_end, align)) rc = DS_EGAP;
      }
      if (rc == DS_OK) {
        if (p->total_bytes && (order.empty() || desc[order[0]].file_offset > 0)) {
          DsTile hole;  // the image starts with bytes of no shard: a tile of pure padding
          std::memset(&hole, 0, sizeof(hole));
          p->tiles.push_back(hole);
          p->tile_off.push_back(0);
        }
        for (size_t k = 0; k < order.size(); ++k) {
          DsTile t = make_tile(desc[order[k]], sizes[order[k]]);
          if (t.n_outer) ++p->n_strided;
          p->tiles.push_back(t);
          p->tile_off.push_back(desc[order[k]].file_offset);
        }
        p->tile_off.push_back(p->total_bytes);
        // the general path's compact copy of the tiles
        p->hot.resize(p->tiles.size() + 1);
        for (size_t t = 0; t <= p->tiles.size(); ++t) {
          DsTileHot &h = p->hot[t];
          std::memset(&h, 0, sizeof(h));
          h.img_off = p->tile_off[t];
          if (t == p->tiles.size()) break;  // the sentinel
          const DsTile &tl = p->tiles[t];
          h.src = tl.src;
          h.nbytes = tl.nbytes;
          uint32_t n_outer = tl.n_outer;
          if (n_outer == 1) {
            h.stride0 = tl.stride[0];
            if (tl.run_bytes < ((uint64_t)1 << 31)) h.run = (uint32_t)tl.run_bytes;
            else n_outer = 2;
          }
          h.meta = n_outer | (tl.es_log2 << 8);
        }
        const uint64_t chunk = ds_cfg_chunk_bytes();
        p->chunk_log2 = (uint32_t)__builtin_ctzll(chunk);
        const uint64_t n_chunks = (p->total_bytes + chunk - 1) >> p->chunk_log2;
        if (n_chunks >= 0x7FFFFFFFull || p->tiles.size() >= 0x7FFFFFFFull) rc = DS_EINVAL;
        if (rc == DS_OK) {
          p->first_tile.resize(n_chunks + 1);
          size_t t = 0;  // tile that holds image byte c*chunk
          for (uint64_t c = 0; c < n_chunks; ++c) {
            const uint64_t at = c << p->chunk_log2;
            while (p->tile_off[t + 1] <= at) ++t;
            p->first_tile[c] = (uint32_t)t;
          }
          p->first_tile[n_chunks] = (uint32_t)p->tiles.size();
          // classify every chunk for the kernel's lean path
          p->recs.resize(n_chunks);
          for (uint64_t c = 0; c < n_chunks; ++c) {
            DsChunkRec &r = p->recs[c];
            std::memset(&r, 0, sizeof(r));
            const uint64_t cb = c << p->chunk_log2, ce = cb + chunk;
            const uint32_t ti = p->first_tile[c];
            const DsTile &tl = p->tiles[ti];
            const uint64_t tb = p->tile_off[ti];
            r.tile = ti;
            r.kind = DS_CHUNK_GENERAL;
            // simple = the whole chunk is whole 16-byte units of ONE tile's payload
            if (ce <= p->total_bytes && ce <= tb + (tl.nbytes & ~(uint64_t)15)) {
              const uint64_t b0 = cb - tb;
              if (tl.n_outer == 0) {
                r.kind = DS_CHUNK_CONTIG;
                r.addr = tl.src + b0;
                // an interior chunk of a tensor at an odd address: the gather may load aligned units
                if (ds_cfg_variant() != 4 && (r.addr & 15) && b0 >= 16 && b0 + chunk + 16 <= tl.nbytes)
                  r.kind |= DS_CHUNK_REALIGN;
              } else if (tl.n_outer == 1 && tl.run_bytes >= 16 && tl.run_bytes < ((uint64_t)1 << 31)) {
                const uint64_t row0 = b0 / tl.run_bytes;
                r.kind = DS_CHUNK_ROWS | (tl.es_log2 << 8);
                r.addr = tl.src + row0 * tl.stride[0];
                r.pitch = tl.stride[0];
                r.col0 = (uint32_t)(b0 - row0 * tl.run_bytes);
                r.run = (uint32_t)tl.run_bytes;
                // a thread's units are 256 threads x 16 bytes apart: that step, divided by the run
                // length once here instead of once per unit in the kernel
                const uint64_t step = 4096;
                r.tile = (uint32_t)(((step / tl.run_bytes) << 16) | (step % tl.run_bytes));
              }
            }
            if ((r.kind & 0xFF) == DS_CHUNK_GENERAL) {
              // the tiles the chunk holds, so that the kernel is one load away from them
              uint32_t t1 = p->first_tile[c + 1];
              const uint64_t c_end = std::min(ce, p->total_bytes);
              if (p->tile_off[t1] >= c_end) --t1;  // that tile starts where this chunk ends
              r.col0 = t1 - ti;
              ++p->n_general;
            }
          }
        }
      }
    }
  } catch (const std::bad_alloc &) {
    rc = DS_ENOMEM;
  }
  if (rc == DS_OK && !(flags & DS_PLAN_HOST_ONLY)) rc = upload(p);
  if (rc != DS_OK) {
    if (p->dev_blob) (void)hipFree(p->dev_blob);
    delete p;
    return rc;
  }
  *out = p;
  return DS_OK;
}

int ds_plan_destroy(ds_plan *plan) {
  if (!plan) return DS_EINVAL;
  int rc = DS_OK;
  if (plan->dev_blob) {
    hipError_t e = hipFree(plan->dev_blob);
    if (e != hipSuccess) { ds_set_hip_error(e); rc = DS_EHIP; }
  }
  delete plan;
  return rc;
}

int ds_plan_info(const ds_plan *plan, ds_plan_stats *out) {
  if (!plan || !out) return DS_EINVAL;
  out->total_bytes = plan->total_bytes;
  out->payload_bytes = plan->payload_bytes;
  out->n_shards = plan->n_shards;
  out->n_tiles = plan->tiles.size();
  out->n_chunks = plan->n_chunks();
  out->chunk_bytes = (uint64_t)1 << plan->chunk_log2;
  out->n_strided = plan->n_strided;
  out->n_general_chunks = plan->n_general;
  out->align = plan->align;
  out->n_files = plan->file_begin.size() - 1;
  return DS_OK;
}

int ds_plan_file(const ds_plan *plan, uint32_t f, uint64_t *image_begin, uint64_t *region_bytes) {
  if (!plan || (size_t)f + 1 >= plan->file_begin.size()) return DS_EINVAL;
  if (image_begin) *image_begin = plan->file_begin[f];
  if (region_bytes) *region_bytes = plan->file_begin[f + 1] - plan->file_begin[f];
  return DS_OK;
}

int ds_plan_shard_file(const ds_plan *plan, size_t i, uint32_t *file, uint64_t *image_offset) {
  if (!plan || i >= plan->manifest.size()) return DS_EINVAL;
  if (file) *file = plan->manifest[i].file;
  if (image_offset) *image_offset = plan->manifest[i].image_offset;
  return DS_OK;
}

int ds_plan_shard(const ds_plan *plan, size_t i, uint64_t *tensor_id, uint32_t *dtype, uint64_t *file_offset,
                  uint64_t *nbytes) {
  if (!plan || i >= plan->manifest.size()) return DS_EINVAL;
  const DsManifestEntry &m = plan->manifest[i];
  if (tensor_id) *tensor_id = m.tensor_id;
  if (dtype) *dtype = m.dtype;
  if (file_offset) *file_offset = m.file_offset;
  if (nbytes) *nbytes = m.nbytes;
  return DS_OK;
}

int ds_plan_shard_shape(const ds_plan *plan, size_t i, uint32_t *ndim, int64_t *shape) {
  if (!plan || i >= plan->manifest.size()) return DS_EINVAL;
  const DsManifestEntry &m = plan->manifest[i];
  if (ndim) *ndim = m.ndim;
  if (shape)
    for (uint32_t j = 0; j < DS_MAX_DIMS; ++j) shape[j] = m.shape[j];
  return DS_OK;
}

int ds_pack(const ds_plan *plan, void *dst_dev, uint64_t img_lo, uint64_t img_hi, void *stream) {
  if (!plan || !plan->dev_blob) return DS_EINVAL;
  if (img_lo > img_hi || img_hi > plan->total_bytes || ((img_lo | img_hi) & 15)) return DS_ERANGE;
  if (img_lo == img_hi) return DS_OK;
  if (!dst_dev || ((uintptr_t)dst_dev & 15)) return DS_EINVAL;
  return ds_launch_move(plan, true, (uint8_t *)dst_dev, img_lo, img_hi, (uint32_t)g_grid_limit.load(), (hipStream_t)stream);
}

int ds_unpack(const ds_plan *plan, const void *src_dev, uint64_t img_lo, uint64_t img_hi, void *stream) {
  if (!plan || !plan->dev_blob) return DS_EINVAL;
  if (img_lo > img_hi || img_hi > plan->total_bytes || ((img_lo | img_hi) & 15)) return DS_ERANGE;
  if (img_lo == img_hi) return DS_OK;
  if (!src_dev || ((uintptr_t)src_dev & 15)) return DS_EINVAL;
  return ds_launch_move(plan, false, (uint8_t *)src_dev, img_lo, img_hi, (uint32_t)g_grid_limit.load(), (hipStream_t)stream);
}

}  // extern "C"
