/*
 * ds_oracle.c -- plain CPU reference for the snapshot image of one GPU's shards.
 *
 * TEST INFRASTRUCTURE ONLY.  This file defines what the packed checkpoint image
 * of a shard table is, in the most literal way available, so that the HIP
 * library can be compared against it byte for byte.  Only the tests, the smoke
 * check and the CPU-baseline leg of the benchmark may build, load or call it.
 * It shares no code, header or table with the HIP library: the descriptor
 * struct below is declared here on purpose, not included.
 *
 * What it follows (DataStates-LLM, arXiv 2601.16956):
 *   - Sec. IV-D and Sec. V-A3: a tensor needs no serialisation; its bytes are
 *     written as they are (no dtype conversion, no byte swap).
 *   - Sec. V-A5, rule (1): tensor sizes are known in advance, hence the offset
 *     of every tensor in the file is precomputed from the sizes alone.
 *   - Sec. V-A1: all shards of one checkpoint are coalesced into one
 *     pre-allocated region.
 * Readings where the paper is silent (all listed in the design notes of the
 * repository): a strided view is stored in row-major order of the VIEW, last
 * index fastest; bytes of the image that belong to no shard are 0x00; the image
 * length is rounded up to the alignment.
 *
 * Pinned by tests/test_oracle_pins.py (hand-computed layouts, closed-form
 * index-encoded images, numpy.tobytes() for contiguous shards, an independent
 * brute-force numpy twin, round-trip and sentinel invariants).
 */
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define DSO_MAX_DIMS 6

enum { DSO_F32 = 0, DSO_BF16 = 1, DSO_F16 = 2, DSO_I64 = 3, DSO_U8 = 4 };

enum {
  DSO_OK = 0,
  DSO_BAD_ARG = -1,     /* unknown dtype, ndim too large, negative extent   */
  DSO_BAD_ALIGN = -2,   /* an offset is not a multiple of the alignment      */
  DSO_OVERLAP = -3,     /* two shards' byte ranges in the image intersect    */
  DSO_GAP = -4,         /* a hole that is not alignment padding              */
  DSO_OUT_OF_IMAGE = -5 /* a shard does not fit into the image length given  */
};

typedef struct {
  void *base;                     /* host address of element (0,...,0)       */
  uint32_t dtype;                 /* DSO_*                                   */
  uint32_t ndim;                  /* 0..6; 0 means exactly one element       */
  int64_t shape[DSO_MAX_DIMS];
  int64_t strides[DSO_MAX_DIMS];  /* in elements                             */
  uint64_t tensor_id;             /* carried along; never touches the bytes  */
  uint64_t file_offset;           /* byte offset of the shard in the image   */
} dso_shard;

int dso_itemsize(uint32_t dtype) {
  switch (dtype) {
    case DSO_F32: return 4;
    case DSO_BF16: return 2;
    case DSO_F16: return 2;
    case DSO_I64: return 8;
    case DSO_U8: return 1;
    default: return 0;
  }
}

/* number of elements = product of the extents; the empty product is 1 */
static int64_t shard_elems(const dso_shard *d) {
  int64_t n = 1;
  for (uint32_t j = 0; j < d->ndim; ++j) n *= d->shape[j];
  return n;
}

static int shard_ok(const dso_shard *d) {
  if (dso_itemsize(d->dtype) == 0 || d->ndim > DSO_MAX_DIMS) return 0;
  for (uint32_t j = 0; j < d->ndim; ++j)
    if (d->shape[j] < 0) return 0;
  return 1;
}

/* packed size of a shard in bytes: itemsize x number of elements */
int64_t dso_shard_bytes(const dso_shard *d) {
  if (!shard_ok(d)) return DSO_BAD_ARG;
  return (int64_t)dso_itemsize(d->dtype) * shard_elems(d);
}

static uint64_t round_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

/*
 * Canonical layout (Sec. V-A5 rule (1)): shards in table order, each at the
 * next multiple of `align` after the end of the one before; the image ends at
 * a multiple of `align` too.  Writes file_offset of every entry.
 */
int dso_layout(dso_shard *d, size_t n, uint64_t align, uint64_t *total) {
  if (align == 0) return DSO_BAD_ARG;
  uint64_t at = 0;
  for (size_t i = 0; i < n; ++i) {
    int64_t b = dso_shard_bytes(&d[i]);
    if (b < 0) return DSO_BAD_ARG;
    d[i].file_offset = at;
    at = round_up(at + (uint64_t)b, align);
  }
  *total = at;
  return DSO_OK;
}

/* image length for offsets that are already given: end of the last byte of
 * any shard (or the offset of an empty one), rounded up to the alignment */
int dso_image_bytes(const dso_shard *d, size_t n, uint64_t align, uint64_t *total) {
  if (align == 0) return DSO_BAD_ARG;
  uint64_t end = 0;
  for (size_t i = 0; i < n; ++i) {
    int64_t b = dso_shard_bytes(&d[i]);
    if (b < 0) return DSO_BAD_ARG;
    if (d[i].file_offset + (uint64_t)b > end) end = d[i].file_offset + (uint64_t)b;
  }
  *total = round_up(end, align);
  return DSO_OK;
}

/*
 * Layout invariants, checked pair by pair (quadratic on purpose: no sorting,
 * nothing clever).  With strict != 0 a hole is accepted only if it is the
 * padding between the end of a shard and the next multiple of `align`.
 */
int dso_check_layout(const dso_shard *d, size_t n, uint64_t align, uint64_t total, int strict) {
  if (align == 0) return DSO_BAD_ARG;
  for (size_t i = 0; i < n; ++i) {
    int64_t b = dso_shard_bytes(&d[i]);
    if (b < 0) return DSO_BAD_ARG;
    if (d[i].file_offset % align != 0) return DSO_BAD_ALIGN;
    if (d[i].file_offset + (uint64_t)b > total) return DSO_OUT_OF_IMAGE;
  }
  for (size_t i = 0; i < n; ++i) {
    uint64_t bi = (uint64_t)dso_shard_bytes(&d[i]);
    if (bi == 0) continue;
    for (size_t k = i + 1; k < n; ++k) {
      uint64_t bk = (uint64_t)dso_shard_bytes(&d[k]);
      if (bk == 0) continue;
      uint64_t lo = d[i].file_offset > d[k].file_offset ? d[i].file_offset : d[k].file_offset;
      uint64_t hi_i = d[i].file_offset + bi, hi_k = d[k].file_offset + bk;
      uint64_t hi = hi_i < hi_k ? hi_i : hi_k;
      if (lo < hi) return DSO_OVERLAP;
    }
  }
  if (strict) {
    /* every byte of [0,total) must lie in a shard or in that shard's padding
     * up to the next multiple of align: walk the multiples of align */
    if (total % align != 0) return DSO_GAP;
    for (uint64_t blk = 0; blk < total; blk += align) {
      int covered = 0;
      for (size_t i = 0; i < n && !covered; ++i) {
        uint64_t b = (uint64_t)dso_shard_bytes(&d[i]);
        if (b == 0) continue;
        uint64_t lo = d[i].file_offset, hi = round_up(lo + b, align);
        if (lo <= blk && blk < hi) covered = 1;
      }
      if (!covered) return DSO_GAP;
    }
  }
  return DSO_OK;
}

/*
 * One shard, one direction.  Visits the elements of the view in row-major
 * order (last index fastest).  Element number r (counted in that order) lives
 * at   base + itemsize * sum_j k_j * strides[j]   in the tensor and at
 * image + file_offset + r * itemsize   in the image.
 * to_image != 0: tensor -> image (pack); else image -> tensor (unpack).
 * When the last stride is 1 a whole innermost row is one memcpy; that is the
 * same bytes in the same places as the element loop below it.
 */
static void copy_shard(const dso_shard *d, uint8_t *image, int to_image) {
  const int64_t es = dso_itemsize(d->dtype);
  const int64_t total = shard_elems(d);
  if (total == 0) return;
  uint8_t *img = image + d->file_offset;
  uint8_t *base = (uint8_t *)d->base;
  const uint32_t nd = d->ndim;
  if (nd == 0) {
    if (to_image) memcpy(img, base, (size_t)es); else memcpy(base, img, (size_t)es);
    return;
  }
  int64_t k[DSO_MAX_DIMS] = {0, 0, 0, 0, 0, 0};
  const int64_t inner = d->shape[nd - 1];
  const int64_t inner_stride = d->strides[nd - 1];
  int64_t r = 0; /* rank of element (k_0, ..., k_{nd-2}, 0) */
  for (;;) {
    int64_t pos = 0; /* element position of (k_0..k_{nd-2}, 0) in the tensor */
    for (uint32_t j = 0; j + 1 < nd; ++j) pos += k[j] * d->strides[j];
    uint8_t *row_t = base + es * pos;
    uint8_t *row_i = img + es * r;
    if (inner_stride == 1) {
      if (to_image) memcpy(row_i, row_t, (size_t)(es * inner));
      else memcpy(row_t, row_i, (size_t)(es * inner));
    } else {
      for (int64_t c = 0; c < inner; ++c) {
        uint8_t *et = row_t + es * c * inner_stride;
        uint8_t *ei = row_i + es * c;
        if (to_image) memcpy(ei, et, (size_t)es); else memcpy(et, ei, (size_t)es);
      }
    }
    r += inner;
    /* advance the outer indices like an odometer */
    int j = (int)nd - 2;
    while (j >= 0) {
      if (++k[j] < d->shape[j]) break;
      k[j] = 0;
      --j;
    }
    if (j < 0) break;
  }
}

static int table_fits(const dso_shard *d, size_t n, uint64_t total) {
  for (size_t i = 0; i < n; ++i) {
    int64_t b = dso_shard_bytes(&d[i]);
    if (b < 0) return DSO_BAD_ARG;
    if (d[i].file_offset + (uint64_t)b > total) return DSO_OUT_OF_IMAGE;
  }
  return DSO_OK;
}

/* image[0,total) := 0, then every shard's bytes at its offset */
int dso_pack(const dso_shard *d, size_t n, uint8_t *image, uint64_t total) {
  int rc = table_fits(d, n, total);
  if (rc != DSO_OK) return rc;
  memset(image, 0, (size_t)total);
  for (size_t i = 0; i < n; ++i) copy_shard(&d[i], image, 1);
  return DSO_OK;
}

/* every addressed element of every shard := its bytes in the image; nothing
 * else in the tensors' memory is written */
int dso_unpack(const dso_shard *d, size_t n, const uint8_t *image, uint64_t total) {
  int rc = table_fits(d, n, total);
  if (rc != DSO_OK) return rc;
  for (size_t i = 0; i < n; ++i) copy_shard(&d[i], (uint8_t *)image, 0);
  return DSO_OK;
}

/* ---- the same pack spread over host threads (for the timed CPU baseline) --- */

typedef struct {
  const dso_shard *d;
  size_t n;
  uint8_t *image;
  uint64_t total;
  int tid, nthreads;
} mt_job;

static void *mt_zero(void *p) {
  mt_job *j = (mt_job *)p;
  uint64_t per = (j->total + (uint64_t)j->nthreads - 1) / (uint64_t)j->nthreads;
  uint64_t lo = per * (uint64_t)j->tid;
  uint64_t hi = lo + per < j->total ? lo + per : j->total;
  if (lo < hi) memset(j->image + lo, 0, (size_t)(hi - lo));
  return NULL;
}

static void *mt_copy(void *p) {
  mt_job *j = (mt_job *)p;
  for (size_t i = (size_t)j->tid; i < j->n; i += (size_t)j->nthreads) copy_shard(&j->d[i], j->image, 1);
  return NULL;
}

static int run_threads(mt_job *jobs, int nthreads, void *(*fn)(void *)) {
  pthread_t *th = (pthread_t *)malloc(sizeof(pthread_t) * (size_t)nthreads);
  if (!th) return DSO_BAD_ARG;
  int started = 0;
  for (int t = 0; t < nthreads; ++t) {
    if (pthread_create(&th[t], NULL, fn, &jobs[t]) != 0) break;
    ++started;
  }
  for (int t = 0; t < started; ++t) pthread_join(th[t], NULL);
  /* whatever could not get a thread runs here */
  for (int t = started; t < nthreads; ++t) fn(&jobs[t]);
  free(th);
  return DSO_OK;
}

/* Same result as dso_pack.  Thread t zeroes the t-th slice of the image, then
 * (after all zeroing is done) copies shards t, t+nthreads, ...  Shards do not
 * overlap in the image, so the copies do not race. */
int dso_pack_mt(const dso_shard *d, size_t n, uint8_t *image, uint64_t total, int nthreads) {
  int rc = table_fits(d, n, total);
  if (rc != DSO_OK) return rc;
  if (nthreads < 1) nthreads = 1;
  mt_job *jobs = (mt_job *)malloc(sizeof(mt_job) * (size_t)nthreads);
  if (!jobs) return DSO_BAD_ARG;
  for (int t = 0; t < nthreads; ++t) {
    jobs[t].d = d; jobs[t].n = n; jobs[t].image = image; jobs[t].total = total;
    jobs[t].tid = t; jobs[t].nthreads = nthreads;
  }
  rc = run_threads(jobs, nthreads, mt_zero);
  if (rc == DSO_OK) rc = run_threads(jobs, nthreads, mt_copy);
  free(jobs);
  return rc;
}

size_t dso_sizeof_shard(void) { return sizeof(dso_shard); }
