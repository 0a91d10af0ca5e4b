// Gather (pack) and scatter (unpack) kernels for gfx950.
//
// The image is cut into chunks of 2^chunk_log2 bytes; one work-group moves one
// chunk (DataStates-LLM Sec. V-A1 coalesces the shards of a checkpoint into
// one region; Sec. V-A4: a chunk need not be a whole tensor).  Work is laid
// out in DESTINATION space: thread -> 16-byte unit of the image, so image
// accesses are aligned, contiguous 16-byte vector accesses whatever the
// shards look like, and every work-group moves the same number of bytes
// however fragmented its part of the image is.
//
// One kernel, ds_move_kernel, serves a pack (or unpack) call; a work-group takes one chunk down one of
// two paths:
//
// lean path: one pass per chunk, a chunk being exactly threads x unroll
//   units (16 KiB by default), so a thread issues all its loads, then all its
//   stores, and is done.  Measured on MI355X a plain copy of this shape runs
//   at ~6 TB/s (read+write) against ~5.3 TB/s for work-groups that stream
//   through 64-256 KiB each: many short-lived work-groups keep the addresses
//   in flight inside a compact, moving window of HBM.  Everything the path
//   needs for a chunk is one 32-byte record prepared by the plan (DsChunkRec),
//   so the only dependent load before the data is that record.  It handles the
//   chunks that are whole units of one tile (contiguous, or rows of a 2-D view
//   of at least 16 bytes each).
//
// general path: the remaining chunks (tile boundaries, payload tails, padding,
//   N-D views); their record names the tiles they hold.  The tiles are taken
//   64 at a time: the first wavefront reads one tile's compact descriptor
//   (DsTileHot, 40 bytes) per lane, a wavefront inclusive scan over the unit
//   counts turns the 64 tiles into one dense index space, and the threads of
//   the work-group share that space evenly, four units each per pass, in three
//   phases: (1) registers and LDS only: find the tile of each unit by binary
//   search over the scan and classify it; (2) all loads, nothing between
//   them; (3) all stores.  Large pieces of views with several outer dimensions
//   are taken out of the scan and walked by the whole work-group ("direct").
//
// Tensor-side addresses are only element-aligned.  gfx950 runs with unaligned
// global access enabled, so a 16-byte unit that lies inside one contiguous run
// is one (possibly unaligned) dwordx4 access; a unit that is cut by the end of
// a run or of the payload is assembled from 16-byte loads that lie inside the
// runs (gather), stored in pieces that cover exactly its bytes (scatter), or,
// for runs shorter than 16 bytes, moved element by element, so no byte outside
// the described views is ever read or written.

#include <mutex>

#include "ds_internal.h"
#include "ds_splice.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef u32x4 u32x4_unaligned __attribute__((aligned(1)));

constexpr int kWave = 64;
constexpr uint32_t kBigUnits = 512;       // N-D views: pieces of >= 8 KiB inside a chunk leave the scan

struct MoveArgs {
  const DsTile *tiles;
  const DsTileHot *hot;  // n_tiles + 1 entries: the general path's compact copy of the tiles, and a sentinel
  const uint32_t *first_tile;
  uint8_t *img;         // points at image byte img_lo
  uint64_t img_lo, img_hi;
  uint64_t total;       // image length
  uint32_t chunk_log2;
  uint32_t n_extra;     // 0..2 chunks cut by img_lo / img_hi: they take the general path whatever their kind
  uint32_t extra[2];
};

struct LeanArgs {
  const DsChunkRec *recs;
  uint8_t *img;        // points at image byte img_lo
  uint64_t img_lo;
  uint32_t chunk_log2;
  uint32_t c_lo;       // first whole chunk inside [img_lo, img_hi)
  uint32_t n_chunks;   // whole chunks inside the range
  uint32_t xcd_span;   // chunks per XCD (ceil(n_chunks / 8)); 0 = work-group i takes chunk i
};

// ---- 16-byte accesses -------------------------------------------------------
// Every address here is device (or pinned host) memory reached through the global address space; saying so
// makes the compiler emit global_load / global_store instead of the flat forms, which also have to ask
// whether the address lies in LDS or scratch.
#define DS_GLOBAL __attribute__((address_space(1)))
template <bool NT>
__device__ __forceinline__ u32x4 ld16_aligned(const uint8_t *p) {
  if (NT) return __builtin_nontemporal_load((const DS_GLOBAL u32x4 *)p);
  return *(const DS_GLOBAL u32x4 *)p;
}
template <bool NT>
__device__ __forceinline__ void st16_aligned(uint8_t *p, u32x4 v) {
  if (NT) __builtin_nontemporal_store(v, (DS_GLOBAL u32x4 *)p);
  else *(DS_GLOBAL u32x4 *)p = v;
}
template <bool NT>
__device__ __forceinline__ u32x4 ld16_any(const uint8_t *p) {
  if (NT) return __builtin_nontemporal_load((const DS_GLOBAL u32x4_unaligned *)p);
  return *(const DS_GLOBAL u32x4_unaligned *)p;
}
template <bool NT>
__device__ __forceinline__ void st16_any(uint8_t *p, u32x4 v) {
  if (NT) __builtin_nontemporal_store(v, (DS_GLOBAL u32x4_unaligned *)p);
  else *(DS_GLOBAL u32x4_unaligned *)p = v;
}

// ---- index arithmetic -------------------------------------------------------
__device__ __forceinline__ void divmod(uint64_t a, uint64_t b, uint64_t &q, uint64_t &r) {
  if (((a | b) >> 32) == 0) {
    uint32_t qq = (uint32_t)a / (uint32_t)b;
    q = qq;
    r = (uint32_t)a - qq * (uint32_t)b;
  } else {
    q = a / b;
    r = a - q * b;
  }
}

// address of the first byte of run number `row` (runs counted in row-major
// order of the outer dimensions)
__device__ __forceinline__ uint64_t run_address(const DsTile *t, uint64_t row) {
  const uint32_t m = t->n_outer;
  if (m == 0) return t->src;
  if (m == 1) return t->src + row * t->stride[0];
  uint64_t a = t->src;
  for (int j = (int)m - 1; j > 0; --j) {
    uint64_t q, r;
    divmod(row, t->extent[j], q, r);
    a += r * t->stride[j];
    row = q;
  }
  return a + row * t->stride[0];
}

// ---- element-wise move of (part of) one unit, exact bounds -------------------
template <int ES> struct ElemType;
template <> struct ElemType<1> { typedef uint8_t type; };
template <> struct ElemType<2> { typedef uint16_t type; };
template <> struct ElemType<4> { typedef uint32_t type; };
template <> struct ElemType<8> { typedef uint64_t type; };

union Unit {
  u32x4 q;
  uint8_t b[16];
  uint16_t h[8];
  uint32_t w[4];
  uint64_t d[2];
};

template <int ES> __device__ __forceinline__ typename ElemType<ES>::type unit_get(const Unit &u, int e);
template <> __device__ __forceinline__ uint8_t unit_get<1>(const Unit &u, int e) { return u.b[e]; }
template <> __device__ __forceinline__ uint16_t unit_get<2>(const Unit &u, int e) { return u.h[e]; }
template <> __device__ __forceinline__ uint32_t unit_get<4>(const Unit &u, int e) { return u.w[e]; }
template <> __device__ __forceinline__ uint64_t unit_get<8>(const Unit &u, int e) { return u.d[e]; }
template <int ES> __device__ __forceinline__ void unit_set(Unit &u, int e, typename ElemType<ES>::type x);
template <> __device__ __forceinline__ void unit_set<1>(Unit &u, int e, uint8_t x) { u.b[e] = x; }
template <> __device__ __forceinline__ void unit_set<2>(Unit &u, int e, uint16_t x) { u.h[e] = x; }
template <> __device__ __forceinline__ void unit_set<4>(Unit &u, int e, uint32_t x) { u.w[e] = x; }
template <> __device__ __forceinline__ void unit_set<8>(Unit &u, int e, uint64_t x) { u.d[e] = x; }

// Moves the first `valid` bytes (a multiple of ES, <= 16) of a unit whose first
// byte is byte `col` of run `row`.  PACK: tensor -> val (rest stays 0);
// else val -> tensor.
template <int ES, bool PACK>
__device__ __forceinline__ void move_elements(const DsTile *t, uint64_t row, uint64_t col, uint32_t valid, Unit &val) {
  typedef typename ElemType<ES>::type E;
  const uint64_t L = t->run_bytes;
  uint64_t ra = run_address(t, row);
#pragma unroll
  for (int e = 0; e < 16 / ES; ++e) {
    if ((uint32_t)(e * ES) < valid) {
      if (col >= L) {  // the run ended exactly here: go on in the next one
        col = 0;
        ++row;
        ra = run_address(t, row);
      }
      E *p = reinterpret_cast<E *>(ra + col);
      if (PACK) unit_set<ES>(val, e, *p);
      else *p = unit_get<ES>(val, e);
      col += ES;
    }
  }
}

// Kept out of line: it is the rare path, and inlining its four instantiations
// at every call site multiplies code size and build time.
// The unit travels by value (in registers), not through the stack.
template <bool PACK>
__device__ __noinline__ u32x4 move_elements_any(const DsTile *t, uint64_t row, uint64_t col, uint32_t valid, u32x4 in) {
  Unit val;
  val.q = in;
  switch (t->es_log2) {
    case 0: move_elements<1, PACK>(t, row, col, valid, val); break;
    case 1: move_elements<2, PACK>(t, row, col, valid, val); break;
    case 2: move_elements<4, PACK>(t, row, col, valid, val); break;
    default: move_elements<8, PACK>(t, row, col, valid, val); break;
  }
  return val.q;
}

// ---- one unit, any tile, any position (the general routine) ------------------
// x: image offset of the unit (multiple of 16) inside tile t's range; imgp: its
// address in the image buffer.
template <bool PACK, bool NTL, bool NTS>
__device__ __forceinline__ void move_unit(const DsTile *t, uint64_t tile_begin, uint64_t x, uint8_t *imgp) {
  const uint64_t nbytes = t->nbytes;
  const uint64_t b = x - tile_begin;
  if (b >= nbytes) {  // padding
    if (PACK) st16_aligned<NTS>(imgp, u32x4{0, 0, 0, 0});
    return;
  }
  const uint64_t left = nbytes - b;
  const uint32_t valid = left < 16 ? (uint32_t)left : 16u;
  const uint64_t L = t->run_bytes;
  uint64_t row = 0, col = b;
  if (t->n_outer) divmod(b, L, row, col);
  if (valid == 16 && col + 16 <= L) {
    uint8_t *p = reinterpret_cast<uint8_t *>(run_address(t, row) + col);
    if (PACK) st16_aligned<NTS>(imgp, ld16_any<NTL>(p));
    else st16_any<NTS>(p, ld16_aligned<NTL>(imgp));
    return;
  }
  if (PACK) st16_aligned<NTS>(imgp, move_elements_any<true>(t, row, col, valid, u32x4{0, 0, 0, 0}));
  else (void)move_elements_any<false>(t, row, col, valid, ld16_aligned<NTL>(imgp));
}

// ---- direct path: one tile range, whole work-group ---------------------------
// [lo, hi): image range of the tile clipped to the chunk, multiples of 16.
template <bool PACK, int NT, int UNROLL, bool NTL, bool NTS>
__device__ __forceinline__ void move_tile_direct(const DsTile *t, uint64_t tile_begin, uint64_t lo, uint64_t hi,
                                                 uint8_t *img, uint64_t img_lo) {
  const uint32_t tid = threadIdx.x;
  const uint64_t nbytes = t->nbytes;
  const uint64_t full_end = tile_begin + (nbytes & ~(uint64_t)15);  // image offset where whole payload units end
  const uint32_t n_all = (uint32_t)((hi - lo) >> 4);
  uint32_t n_full = 0;
  if (full_end > lo) n_full = (uint32_t)(((full_end < hi ? full_end : hi) - lo) >> 4);
  uint8_t *imgp = img + (lo - img_lo);
  const uint64_t b0 = lo - tile_begin;
  const uint32_t m = t->n_outer;

  if (m == 0) {
    uint8_t *s = reinterpret_cast<uint8_t *>(t->src + b0);
    for (uint32_t base = 0; base < n_full; base += NT * UNROLL) {
      u32x4 v[UNROLL];
#pragma unroll
      for (int i = 0; i < UNROLL; ++i) {
        const uint32_t u = base + i * NT + tid;
        if (u < n_full) v[i] = PACK ? ld16_any<NTL>(s + 16ull * u) : ld16_aligned<NTL>(imgp + 16ull * u);
      }
#pragma unroll
      for (int i = 0; i < UNROLL; ++i) {
        const uint32_t u = base + i * NT + tid;
        if (u < n_full) {
          if (PACK) st16_aligned<NTS>(imgp + 16ull * u, v[i]);
          else st16_any<NTS>(s + 16ull * u, v[i]);
        }
      }
    }
  } else {
    const uint64_t L = t->run_bytes;
    uint64_t row0, col0;
    divmod(b0, L, row0, col0);
    if (L < (1ull << 31)) {
      const uint32_t L32 = (uint32_t)L, c32 = (uint32_t)col0;
      for (uint32_t base = 0; base < n_full; base += NT * UNROLL) {
#pragma unroll
        for (int i = 0; i < UNROLL; ++i) {
          const uint32_t u = base + i * NT + tid;
          if (u < n_full) {
            const uint32_t tt = c32 + 16u * u;        // < 2^31 + 2^22
            const uint32_t q = tt / L32;
            const uint32_t col = tt - q * L32;
            const uint64_t row = row0 + q;
            uint8_t *ip = imgp + 16ull * u;
            if (col + 16u <= L32) {
              uint8_t *p = reinterpret_cast<uint8_t *>(run_address(t, row) + col);
              if (PACK) st16_aligned<NTS>(ip, ld16_any<NTL>(p));
              else st16_any<NTS>(p, ld16_aligned<NTL>(ip));
            } else {
              if (PACK) st16_aligned<NTS>(ip, move_elements_any<true>(t, row, col, 16, u32x4{0, 0, 0, 0}));
              else (void)move_elements_any<false>(t, row, col, 16, ld16_aligned<NTL>(ip));
            }
          }
        }
      }
    } else {
      for (uint32_t u = tid; u < n_full; u += NT)
        move_unit<PACK, NTL, NTS>(t, tile_begin, lo + 16ull * u, imgp + 16ull * u);
    }
  }
  // the unit cut by the end of the payload, then padding
  for (uint32_t u = n_full + tid; u < n_all; u += NT)
    move_unit<PACK, NTL, NTS>(t, tile_begin, lo + 16ull * u, imgp + 16ull * u);
}

__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t x, uint32_t lane) {
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    const uint32_t y = __shfl_up(x, d, kWave);
    if (lane >= (uint32_t)d) x += y;
  }
  return x;
}

// ---- units cut by the end of a run ------------------------------------------------------
// bytes [s, s+16) of the 32 bytes a||b, 0 < s < 16 (word selects and byte-aligns, see ds_splice.h)
__device__ __forceinline__ u32x4 splice(u32x4 a, u32x4 b, uint32_t s) {
  const DsWords4 r = ds_splice_words(DsWords4{{a.x, a.y, a.z, a.w}}, DsWords4{{b.x, b.y, b.z, b.w}}, s);
  return u32x4{r.w[0], r.w[1], r.w[2], r.w[3]};
}

// The value lane + 1 of the wavefront holds (the last lane keeps its own): one data-parallel move, "wavefront
// shift left by one".
__device__ __forceinline__ uint32_t lane_above(uint32_t x) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, 0x130, 0xF, 0xF, false);
}

// the low n < 16 bytes of v to p (any alignment), as one store each of 8, 4, 2 and 1 bytes as n has those bits
typedef uint64_t u64_unaligned __attribute__((aligned(1)));
typedef uint32_t u32_unaligned __attribute__((aligned(1)));
typedef uint16_t u16_unaligned __attribute__((aligned(1)));
__device__ __forceinline__ void store_low_bytes(uint8_t *p, u32x4 v, uint32_t n) {
  uint64_t lo = v.x | ((uint64_t)v.y << 32);
  const uint64_t hi = v.z | ((uint64_t)v.w << 32);
  if (n & 8) {
    *(DS_GLOBAL u64_unaligned *)p = lo;
    p += 8;
    lo = hi;
  }
  if (n & 4) {
    *(DS_GLOBAL u32_unaligned *)p = (uint32_t)lo;
    p += 4;
    lo >>= 32;
  }
  if (n & 2) {
    *(DS_GLOBAL u16_unaligned *)p = (uint16_t)lo;
    p += 2;
    lo >>= 16;
  }
  if (n & 1) *(DS_GLOBAL uint8_t *)p = (uint8_t)lo;
}
// bytes [0,k) of v go to p0, bytes [k,valid) to p1 (0 < k < 16, k <= valid <= 16); exactly those bytes are written
__device__ __forceinline__ void store_cut(uint8_t *p0, uint8_t *p1, uint32_t k, u32x4 v, uint32_t valid = 16) {
  store_low_bytes(p0, v, k);
  if (valid > k) store_low_bytes(p1, splice(v, u32x4{0, 0, 0, 0}, k), valid - k);
}

// What a batch of up to 64 tiles of a general chunk needs, staged in LDS by the first wavefront.  Everything
// a unit needs is relative to the start of its tile's range inside the (clipped) chunk, so that the per-unit
// arithmetic is 32-bit: a chunk is at most 32 KiB.
struct GenLds {
  uint32_t incl[kWave];   // inclusive scan of the tiles' unit counts inside the chunk
  uint32_t begin[kWave];  // where a tile's clipped range starts, relative to the chunk's clipped start
  uint32_t rem[kWave];    // payload bytes from there on (clamped to 2^31; 0 = padding only)
  uint32_t run[kWave];    // views with one outer dimension: run length
  uint32_t col0[kWave];   // ... and the position of the clipped start inside its run
  uint32_t meta[kWave];   // n_outer | log2(itemsize) << 8 | kRunGe16 if the runs are at least 16 bytes long
  uint64_t src0[kWave];   // address of the clipped start (one run), or of the start of the run that holds it
  uint64_t pitch[kWave];  // views with one outer dimension: distance between runs
  uint64_t big_mask;      // tiles taken out of the scan (large pieces of views with several outer dimensions)
  uint32_t n_units;       // units of the batch = incl[63]
};
constexpr uint32_t kRunGe16 = 1u << 16;
constexpr int kStorePolicySc0Sc1Nt = 1 | 2 | 16;  // sc0 | nt | sc1 in the buffer-store intrinsic's aux operand
// s_waitcnt immediate on gfx9: vmcnt = 0 (bits 3:0 and 15:14), expcnt (6:4) and lgkmcnt (11:8) left at their maxima
constexpr int kWaitVmcnt0 = 0x0F70;

// One general chunk, whole work-group: chunk number c, which holds (parts of) tiles t0 .. t1.
//
// The tiles are taken 64 at a time.  The first wavefront reads their compact descriptors (DsTileHot, one tile
// per lane), turns the unit counts into one dense index space with an inclusive scan, and leaves what the
// units need in LDS; then every thread takes the units tid, tid + NT, ... of that space, UNROLL at a time in
// phases: find the tile of each unit (binary search over the scan) and classify it, issue all loads, issue
// all stores.  So a chunk costs three dependent trips to memory (record -> descriptors -> data) however many
// tiles it holds.  Units that are one 16-byte access (inside the payload of a contiguous tile or inside a row
// of a 2-D view), padding, and units cut by the end of a run of at least 16 bytes are handled in the phases;
// only the rest (runs shorter than 16 bytes, views with several outer dimensions) goes one by one through
// move_unit afterwards.
template <bool PACK, int NT, int UNROLL, bool NTL, bool NTS, bool BUFST>
__device__ __forceinline__ void general_chunk(const MoveArgs &a, uint64_t c, uint32_t t0, uint32_t t1, GenLds *g) {
  const uint32_t tid = threadIdx.x;
  const uint32_t lane = tid & (kWave - 1);
  const uint64_t c_begin = c << a.chunk_log2;
  uint64_t c_end = (c + 1) << a.chunk_log2;
  if (c_end > a.total) c_end = a.total;
  const uint64_t cb = c_begin > a.img_lo ? c_begin : a.img_lo;
  const uint64_t ce = c_end < a.img_hi ? c_end : a.img_hi;
  if (cb >= ce) return;
  uint8_t *const cimg = a.img + (cb - a.img_lo);  // the chunk's (clipped) start in the image buffer
  // Gather with buffer stores: the resource covers exactly the chunk's part of the image, and a lane that has
  // nothing to store in a phase gives an offset beyond it, which the hardware drops.  The stores of a phase
  // are then plain instructions one behind the other, with no branch (and no wait) between them.
  __amdgpu_buffer_rsrc_t image_rsrc;
  if (PACK && BUFST) image_rsrc = __builtin_amdgcn_make_buffer_rsrc(cimg, 0, (int)(uint32_t)(ce - cb), 0x00020000);
  constexpr uint32_t kNoStore = 0x80000000u;

  for (uint32_t bt = t0; bt <= t1; bt += kWave) {
    __syncthreads();  // readers of the previous batch (or of the previous chunk) are done
    if (tid < kWave) {
      const uint32_t ti = bt + lane;
      uint64_t lo = cb, hi = cb, tb = cb;
      uint64_t src = 0, nbytes = 0, stride0 = 0;
      uint32_t run = 0, meta = 0;
      if (ti <= t1) {
        const DsTileHot *h = a.hot + ti;
        tb = h->img_off;
        src = h->src;
        nbytes = h->nbytes;
        stride0 = h->stride0;
        run = h->run;
        meta = h->meta;
        const uint64_t te = h[1].img_off;  // the entry behind the last tile is a sentinel
        lo = tb > cb ? tb : cb;
        hi = te < ce ? te : ce;
        if (hi < lo) hi = lo;
      }
      const uint32_t n_outer = meta & 0xFFu;
      const uint32_t units = (uint32_t)((hi - lo) >> 4);
      const bool big = units >= kBigUnits && n_outer > 1;
      const uint64_t big_mask = __ballot(big);
      const uint32_t incl = wave_inclusive_scan(big ? 0u : units, lane);
      const uint64_t b0 = lo - tb;  // byte of the tile's own range at which its clipped range starts
      uint64_t rem = b0 < nbytes ? nbytes - b0 : 0;
      if (rem > (1ull << 31)) rem = 1ull << 31;
      uint64_t src0 = src + b0;
      uint32_t col0 = 0;
      uint64_t longest = nbytes;  // length of the tile's runs
      if (n_outer == 1) {
        uint64_t row0, c0;
        divmod(b0, run, row0, c0);
        src0 = src + row0 * stride0;
        col0 = (uint32_t)c0;
        longest = run;
      }
      g->incl[lane] = incl;
      g->begin[lane] = (uint32_t)(lo - cb);
      g->rem[lane] = (uint32_t)rem;
      g->run[lane] = run;
      g->col0[lane] = col0;
      g->meta[lane] = meta | (longest >= 16 ? kRunGe16 : 0u);
      g->src0[lane] = src0;
      g->pitch[lane] = stride0;
      if (lane == kWave - 1) {
        g->n_units = incl;
        g->big_mask = big_mask;
      }
    }
    __syncthreads();
    const uint32_t n_units = g->n_units;
    for (uint32_t base = 0; base < n_units; base += NT * UNROLL) {
      // how[i]: kind | k << 8 | last << 16 | tile << 24 (k: bytes of a cut unit that end its run; last: the
      // payload ends with that run; tile: 0..63 inside the batch)
      enum : uint32_t { kNone = 0, kFast = 1, kZero = 2, kCut = 3, kSlow = 4, kCutHeld = 5, kKind = 0xFFu, kLast = 1u << 16 };
      uint32_t j[UNROLL], p[UNROLL], how[UNROLL];
      uint8_t *ip[UNROLL];   // the unit in the image buffer
      uint8_t *sp[UNROLL];   // kFast, kCut: where the unit starts in the tensor
      // ---- phase 1, registers and LDS only: which tile each unit belongs to, and what kind of unit it is ----
      // A thread's i-th unit of the pass.  Each block of NT units is rotated by 9 more than the one before:
      // tensors of one size put their cut units at a fixed period, and periods that divide NT (slots of 512
      // bytes to 4 KiB) would otherwise give all of them to the same few threads, four each.
#pragma unroll
      for (int i = 0; i < UNROLL; ++i) {
        j[i] = base + i * NT + ((tid + 40u * i) & (NT - 1));
        p[i] = 0;
      }
      // smallest p with incl[p] > j, the searches of the thread's units side by side (a unit beyond the end
      // of the batch ends at tile 63: every index stays inside the table)
#pragma unroll
      for (int step = kWave / 2; step > 0; step >>= 1) {
#pragma unroll
        for (int i = 0; i < UNROLL; ++i)
          if (g->incl[p[i] + step - 1] <= j[i]) p[i] += step;
      }
#pragma unroll
      for (int i = 0; i < UNROLL; ++i) {
        how[i] = kNone;
        ip[i] = cimg;
        sp[i] = cimg;
        if (j[i] < n_units) {
          const uint32_t q = p[i];
          const uint32_t d = 16u * (j[i] - (q ? g->incl[q - 1] : 0u));  // the unit's offset in the tile's clipped range
          ip[i] = cimg + (g->begin[q] + d);
          const uint32_t rem = g->rem[q];
          const uint32_t meta = g->meta[q];
          if (d >= rem) {
            how[i] = kZero;
          } else if ((meta & 0xFFu) > 1 || !(meta & kRunGe16)) {
            how[i] = kSlow | (q << 24);
          } else {
            // the run the unit starts in: what is left of the payload, or one row of a 2-D view
            uint64_t run0 = g->src0[q];
            uint32_t L = rem, col = d;
            if (meta & 0xFFu) {
              L = g->run[q];
              const uint32_t t = g->col0[q] + d;  // < 2^31 + 2^15
              const uint32_t rows = t / L;
              col = t - rows * L;
              run0 += (uint64_t)rows * g->pitch[q];
            }
            sp[i] = reinterpret_cast<uint8_t *>(run0 + col);
            if (col + 16u <= L) {
              how[i] = kFast;
            } else {
              const uint32_t k = L - col;
              // unless the payload ends with this run, the unit goes on in the next one
              const bool last = !(meta & 0xFFu) || d + k >= rem;
              how[i] = kCut | (k << 8) | (last ? kLast : 0u) | (q << 24);
            }
          }
        }
      }
      // Gather: the thread's first cut unit of the pass travels with the others: its two loads are issued in
      // the load phase, it is spliced into v[] and leaves with the same store instruction as its neighbours
      // (so that a line of the image is written whole).  Further cut units of the same thread wait for a
      // phase of their own; the rotation above makes them rare.  (Chosen here, after the units have been
      // classified independently of each other, so that their classifications can run side by side.)
      bool cut_held = false;
      uint8_t *cut_pa = nullptr, *cut_pb = nullptr;  // the last 16 bytes of the run; the first 16 of the next (or null)
      if (PACK) {
#pragma unroll
        for (int i = 0; i < UNROLL; ++i)
          if ((how[i] & kKind) == kCut && !cut_held) {
            cut_held = true;
            const uint32_t k = (how[i] >> 8) & 0xFFu, q = how[i] >> 24;
            cut_pa = sp[i] + k - 16;
            if (!(how[i] & kLast)) cut_pb = sp[i] + k + (g->pitch[q] - g->run[q]);
            how[i] = kCutHeld | (k << 8);
          }
      }
      // ---- phase 2: all loads, nothing between them ----
      u32x4 v[UNROLL];
#pragma unroll
      for (int i = 0; i < UNROLL; ++i) v[i] = u32x4{0, 0, 0, 0};  // padding is written as zeros
      u32x4 cut_a = u32x4{0, 0, 0, 0}, cut_b = u32x4{0, 0, 0, 0};
#pragma unroll
      for (int i = 0; i < UNROLL; ++i) {
        const uint32_t kind = how[i] & kKind;
        if (PACK) {
          if (kind == kFast) v[i] = ld16_any<NTL>(sp[i]);
        } else {
          if (kind == kFast || kind == kCut) v[i] = ld16_aligned<NTL>(ip[i]);
        }
      }
      if (PACK && cut_held) {
        cut_a = ld16_any<NTL>(cut_pa);
        if (cut_pb) cut_b = ld16_any<NTL>(cut_pb);
      }
      // ---- phase 3: all stores ----
      // Every load has landed before the first store goes out.  Loads and stores share one counter and
      // complete out of order with respect to each other, so a wait for a load that is issued behind a store
      // waits for that store as well; left to itself the compiler, which cannot tell on every path that the
      // loads are done, puts such a wait in front of each store and the stores leave one round trip apart.
      __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);
      if (PACK) {
        if (cut_held) {
          uint32_t k = 0;
#pragma unroll
          for (int i = 0; i < UNROLL; ++i)
            if ((how[i] & kKind) == kCutHeld) k = (how[i] >> 8) & 0xFFu;
          const u32x4 spliced = splice(cut_a, cut_b, 16u - k);
#pragma unroll
          for (int i = 0; i < UNROLL; ++i)
            if ((how[i] & kKind) == kCutHeld) v[i] = spliced;
        }
#pragma unroll
        for (int i = 0; i < UNROLL; ++i) {
          const uint32_t kind = how[i] & kKind;
          const bool stores = kind == kFast || kind == kZero || kind == kCutHeld;
          if (BUFST)
            __builtin_amdgcn_raw_buffer_store_b128(v[i], image_rsrc, (int)(stores ? (uint32_t)(ip[i] - cimg) : kNoStore), 0,
                                                   kStorePolicySc0Sc1Nt);
          else if (stores)
            st16_aligned<NTS>(ip[i], v[i]);
        }
      } else {
#pragma unroll
        for (int i = 0; i < UNROLL; ++i) {
          const uint32_t kind = how[i] & kKind;
          if (kind == kFast) {
            st16_any<NTS>(sp[i], v[i]);
          } else if (kind == kCut) {
            // each part as at most four pieces of 8, 4, 2 and 1 bytes: exactly the bytes of the view
            const uint32_t k = (how[i] >> 8) & 0xFFu, q = how[i] >> 24;
            const bool last = how[i] & kLast;
            store_cut(sp[i], sp[i] + k + (g->pitch[q] - g->run[q]), k, v[i], last ? k : 16u);
          }
        }
      }
      // Gather: a thread's further cut units, one after the other: the first k bytes end their run, the rest
      // start the next one or are padding when the payload ends there; both parts come from 16-byte loads
      // that lie wholly inside their runs.
      if (PACK) {
#pragma unroll
        for (int i = 0; i < UNROLL; ++i)
          if ((how[i] & kKind) == kCut) {
            const uint32_t k = (how[i] >> 8) & 0xFFu, q = how[i] >> 24;
            const u32x4 va = ld16_any<NTL>(sp[i] + k - 16);
            u32x4 vb = u32x4{0, 0, 0, 0};
            if (!(how[i] & kLast)) vb = ld16_any<NTL>(sp[i] + k + (g->pitch[q] - g->run[q]));
            st16_aligned<NTS>(ip[i], splice(va, vb, 16u - k));
          }
      }
      // the rare rest (runs shorter than 16 bytes, views with several outer dimensions), one by one
#pragma unroll
      for (int i = 0; i < UNROLL; ++i)
        if ((how[i] & kKind) == kSlow) {
          const uint32_t q = how[i] >> 24;
          const uint64_t tb = a.hot[bt + q].img_off;
          move_unit<PACK, NTL, NTS>(a.tiles + bt + q, tb, cb + (uint64_t)(ip[i] - cimg), ip[i]);
        }
    }
    uint64_t big_mask = g->big_mask;
    while (big_mask) {
      const uint32_t p = (uint32_t)__builtin_ctzll(big_mask);
      big_mask &= big_mask - 1;
      const uint32_t t = bt + p;
      const uint64_t tb = a.hot[t].img_off, te = a.hot[t + 1].img_off;
      const uint64_t lo2 = tb > cb ? tb : cb, hi2 = te < ce ? te : ce;
      move_tile_direct<PACK, NT, UNROLL, NTL, NTS>(a.tiles + t, tb, lo2, hi2, a.img, a.img_lo);
    }
  }
}

// ---- the lean path -----------------------------------------------------------
// BUFST: the gather writes the image through buffer stores with the cache policy "sc0 sc1 nt"
// (write-through, streaming).  Measured on a plain copy of this shape: 6.25 TB/s against 6.07 TB/s with
// "nt" global stores and 5.88 TB/s with plain ones.  The buffer form is used because the compiler has an
// intrinsic with a cache-policy operand for it (and none for global stores); the resource covers exactly
// the work-group's chunk, so an out-of-range store would be dropped by the hardware.

// Number of lean work items of a launch; item ci takes one lean chunk, whole work-group.
__device__ __forceinline__ uint32_t lean_items(const LeanArgs &a) { return a.xcd_span ? a.xcd_span * 8u : a.n_chunks; }

// Work item ci of a launch: moves its chunk if the chunk is lean and returns false; for a general chunk it
// moves nothing, says which chunk and tiles (c, t0, t1) and returns true: the caller sends it down the general
// path (one call site, so that the general path is in the kernel once).
template <bool PACK, int NT, int UNROLL, bool NTL, bool NTS, bool BUFST>
__device__ __forceinline__ bool lean_chunk(const LeanArgs &a, uint32_t ci, uint64_t &c_gen, uint32_t &t0, uint32_t &t1) {
  const uint32_t tid = threadIdx.x;
  {
    // Work-groups are dealt to the 8 XCDs round-robin (work-group i runs on XCD i mod 8).  Chunk
    // numbers are permuted so that each XCD walks ONE contiguous eighth of the range instead of every
    // eighth chunk: measured +1.5 % (7B rank) to +5 % (fragmentation set) on the gather and +4 to +8 %
    // on the scatter.
    uint32_t cm = ci;
    if (a.xcd_span) {
      cm = (ci & 7u) * a.xcd_span + (ci >> 3);
      if (cm >= a.n_chunks) return false;
    }
    const uint32_t c = a.c_lo + cm;
    const DsChunkRec r = a.recs[c];
    const uint32_t kind = r.kind & 0xFF;  // bits 8.. hold log2(itemsize)
    if (kind == DS_CHUNK_GENERAL) {
      // its record names the tiles it holds: one load away from them, and in place among its neighbours
      c_gen = c;
      t0 = r.tile;
      t1 = r.tile + r.col0;
      return true;
    }
    uint8_t *imgp = a.img + (((uint64_t)c << a.chunk_log2) - a.img_lo);
    __amdgpu_buffer_rsrc_t image_rsrc;
    if (PACK && BUFST) image_rsrc = __builtin_amdgcn_make_buffer_rsrc(imgp, 0, NT * UNROLL * 16, 0x00020000);
    u32x4 v[UNROLL];
    if (kind == DS_CHUNK_CONTIG) {
      uint8_t *s = reinterpret_cast<uint8_t *>(r.addr);
      // (the scatter keeps "nt" global stores on the tensor side: the write-through buffer stores that serve
      // the image so well cost it 3 % on the Llama ranks and 10 % on the fragmentation set, measured)
      if (PACK && (r.kind & DS_CHUNK_REALIGN)) {
        // The tensor side is at an odd address: a 16-byte load there costs about twice an aligned one.  Every
        // lane loads the ALIGNED unit that holds the first byte of its image unit and takes the rest from
        // the unit of the lane above it (of the same wavefront: the last lane loads that unit itself); the
        // plan sets the flag only where those units lie inside the tensor.
        const uint32_t m = (uint32_t)r.addr & 15u;
        uint8_t *base = s - m;
        const bool last_lane = (tid & (kWave - 1)) == kWave - 1;
        u32x4 a[UNROLL], e[UNROLL];
#pragma unroll
        for (int i = 0; i < UNROLL; ++i) a[i] = ld16_aligned<NTL>(base + 16u * (i * NT + tid));
#pragma unroll
        for (int i = 0; i < UNROLL; ++i) {
          e[i] = u32x4{0, 0, 0, 0};
          if (last_lane) e[i] = ld16_aligned<NTL>(base + 16u * (i * NT + tid) + 16u);
        }
#pragma unroll
        for (int i = 0; i < UNROLL; ++i) {
          u32x4 up = u32x4{lane_above(a[i].x), lane_above(a[i].y), lane_above(a[i].z), lane_above(a[i].w)};
          if (last_lane) up = e[i];
          v[i] = splice(a[i], up, m);
        }
      } else {
#pragma unroll
        for (int i = 0; i < UNROLL; ++i) {
          const uint32_t off = 16u * (i * NT + tid);
          v[i] = PACK ? ld16_any<NTL>(s + off) : ld16_aligned<NTL>(imgp + off);
        }
      }
#pragma unroll
      for (int i = 0; i < UNROLL; ++i) {
        const uint32_t off = 16u * (i * NT + tid);
        if (PACK && BUFST) __builtin_amdgcn_raw_buffer_store_b128(v[i], image_rsrc, (int)off, 0, kStorePolicySc0Sc1Nt);
        else if (PACK) st16_aligned<NTS>(imgp + off, v[i]);
        else st16_any<NTS>(s + off, v[i]);
      }
    } else {
      // DS_CHUNK_ROWS: runs of r.run >= 16 bytes, r.pitch apart.  A unit that lies in one
      // run is one access.  A unit cut by the end of a run takes its first k bytes from
      // the end of that run and the other 16-k from the start of the next one; on the
      // gather side both come from 16-byte loads that lie wholly inside their runs
      // (the last 16 bytes of the one, the first 16 of the other), so nothing outside
      // the view is read; on the scatter side each part is stored as at most four pieces
      // of 8, 4, 2 and 1 bytes, exactly the bytes of the view.
      uint8_t *p[UNROLL];
      uint32_t cut[UNROLL];  // k, or 0 if the unit is not cut
      u32x4 w[UNROLL];       // gather: the first 16 bytes of the next run, for cut units
      // One division for the thread's first unit; its other units are NT*16 bytes further on each,
      // and the plan has divided that step by the run length already (r.tile = quotient << 16 | rest).
      const uint32_t step_q = r.tile >> 16, step_r = r.tile & 0xFFFFu;
      const uint32_t tt0 = r.col0 + 16u * tid;  // < 2^31 + 2^13
      uint32_t q = tt0 / r.run;
      uint32_t col = tt0 - q * r.run;
#pragma unroll
      for (int i = 0; i < UNROLL; ++i) {
        const uint32_t off = 16u * (i * NT + tid);
        uint8_t *row = reinterpret_cast<uint8_t *>(r.addr + (uint64_t)q * r.pitch);
        p[i] = row + col;
        cut[i] = col + 16u > r.run ? r.run - col : 0u;
        if (PACK) {
          // all loads are issued before any of them is used: no wait inside this loop
          v[i] = ld16_any<NTL>(cut[i] ? row + r.run - 16u : p[i]);
          if (cut[i]) w[i] = ld16_any<NTL>(row + r.pitch);
        } else {
          v[i] = ld16_aligned<NTL>(imgp + off);
        }
        q += step_q;
        col += step_r;
        if (col >= r.run) {
          col -= r.run;
          ++q;
        }
      }
      if (PACK) {
#pragma unroll
        for (int i = 0; i < UNROLL; ++i)
          if (cut[i]) v[i] = splice(v[i], w[i], 16u - cut[i]);
      }
#pragma unroll
      for (int i = 0; i < UNROLL; ++i) {
        const uint32_t off = 16u * (i * NT + tid);
        if (PACK && BUFST) {
          __builtin_amdgcn_raw_buffer_store_b128(v[i], image_rsrc, (int)off, 0, kStorePolicySc0Sc1Nt);
        } else if (PACK) {
          st16_aligned<NTS>(imgp + off, v[i]);
        } else if (cut[i] == 0) {
          st16_any<NTS>(p[i], v[i]);
        } else {
          store_cut(p[i], p[i] + cut[i] + (r.pitch - r.run), cut[i], v[i]);
        }
      }
    }
  }
  return false;
}

// Both paths in one launch: work item i takes whole chunk number i of the range (in the XCD-contiguous
// order) down the path its record names, so a general chunk is moved in place, among its neighbours in the
// image, one record load away from its tiles; the at most two chunks cut by the ends of the range follow
// as work items of their own.  History, measured on the gather: lean kernel then general kernel in two
// launches cost the 7B rank a launch gap plus the general kernel's 9 us (5.78 TB/s in the timed region
// against 6.17 now); the general kernel on a side stream beside the lean one gave the fragmentation set
// 5.30 -> 5.54 TB/s, one launch 5.85 TB/s.
//
// At most 4 waves per SIMD (the attribute makes the compiler pad the register allocation): fewer
// work-groups in flight keep the addresses in a more compact window of HBM.  Measured with the cap at 4
// against 5: gather +0.8 % on the 7B and 70B ranks, -0.8 % on the fragmentation set, scatter +0.5 to +1 %
// everywhere; the scatter, whose own registers would allow 8, loses 5 % there; with 3 or fewer both
// directions lose ~9 %.
//
// A lean chunk is exactly 256 threads x UNROLL x 16 bytes; the general path always works in passes of
// 256 x 4 units.
//
// WAVES = 6 is the instantiation for plans in which most chunks are general (tables of thousands of tiny
// tensors): that path is bound by its chain of dependent loads, not by HBM, and more wavefronts per SIMD hide
// more of it -- five for the gather, whose registers allow no more, six for the scatter (measured on tables
// where every chunk is general: +8 to +10 % both ways with five, another +6 to +10 % for the scatter of tiny
// tensors with six), while the lean path loses 2 to 5 % there.
template <bool PACK, int UNROLL, bool NTL, bool NTS, bool BUFST, int WAVES>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, WAVES))) void ds_move_kernel(LeanArgs la,
                                                                                                     MoveArgs ma) {
  __shared__ GenLds s_gen;
  const uint32_t n_lean = lean_items(la);
  const uint32_t n_iter = n_lean + ma.n_extra;
  for (uint32_t wi = blockIdx.x; wi < n_iter; wi += gridDim.x) {
    uint64_t c = 0;
    uint32_t t0 = 0, t1 = 0;
    bool general = true;
    if (wi < n_lean) {
      general = lean_chunk<PACK, 256, UNROLL, NTL, NTS, BUFST>(la, wi, c, t0, t1);
    } else {
      // a chunk cut by the range: the general path clips to the range, whatever the chunk's kind
      c = ma.extra[wi - n_lean];
      uint64_t c_end = (c + 1) << ma.chunk_log2;
      if (c_end > ma.total) c_end = ma.total;
      t0 = ma.first_tile[c];
      t1 = ma.first_tile[c + 1];
      if (ma.hot[t1].img_off >= c_end) --t1;  // that tile starts where this chunk ends
    }
    if (general) general_chunk<PACK, 256, 4, NTL, NTS, BUFST>(ma, c, t0, t1, &s_gen);
  }
}

template <bool PACK, bool NTL, bool NTS, bool BUFST, int WAVES = 4>
int launch_move(uint32_t chunk_log2, const LeanArgs &la, const MoveArgs &ma, uint32_t grid_limit, hipStream_t stream) {
  uint32_t grid = (la.xcd_span ? la.xcd_span * 8 : la.n_chunks) + ma.n_extra;
  if (grid == 0) return DS_OK;
  if (grid_limit && grid > grid_limit) grid = grid_limit;
#define DS_MOVE(UN) \
  hipLaunchKernelGGL((ds_move_kernel<PACK, UN, NTL, NTS, BUFST, WAVES>), dim3(grid), dim3(256), 0, stream, la, ma)
  switch (chunk_log2) {
    case 13: DS_MOVE(2); break;
    case 14: DS_MOVE(4); break;
    case 15: DS_MOVE(8); break;
    default: return DS_EINVAL;
  }
#undef DS_MOVE
  DS_HIP_TRY(hipGetLastError());
  return DS_OK;
}

// A plain contiguous copy in the lean path's shape (256 threads x 4 units per
// work-group, non-temporal 16-byte accesses): the measured ceiling the gather
// is compared with, and the known-size kernel the HBM counters are scaled by.
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 4))) void ds_copy_probe_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst,
                                                            uint64_t n_units) {
  // the same XCD-contiguous order of work-groups as the lean path
  const uint32_t n_groups = (uint32_t)((n_units + 1023) / 1024), span = (n_groups + 7) / 8;
  const uint32_t g = (blockIdx.x & 7u) * span + (blockIdx.x >> 3);
  if (g >= n_groups) return;
  const uint64_t first = (uint64_t)g * 1024;  // this work-group's 1024 units
  const uint64_t left = n_units - first;
  const uint32_t mine = left < 1024 ? (uint32_t)left : 1024u;
  __amdgpu_buffer_rsrc_t out = __builtin_amdgcn_make_buffer_rsrc(dst + first, 0, (int)(mine * 16u), 0x00020000);
  u32x4 v[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (threadIdx.x + 256u * i < mine) v[i] = __builtin_nontemporal_load(src + first + threadIdx.x + 256 * i);
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (threadIdx.x + 256u * i < mine)
      __builtin_amdgcn_raw_buffer_store_b128(v[i], out, (int)(16u * (threadIdx.x + 256u * i)), 0, kStorePolicySc0Sc1Nt);
}

// ---- which blocks of two images differ ----------------------------------------------------------
__global__ __launch_bounds__(256) void ds_clear_flags_kernel(uint32_t *flags, uint64_t n) {
  const uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) flags[i] = 0;
}

// One work-group compares 1024 units (16 KiB) of the two images, in the lean path's shape and order; a
// wavefront that saw a difference sets the flag of the block its units belong to (a 16 KiB piece never
// straddles two blocks: the block size is a multiple of 16 KiB).
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 4))) void ds_diff_kernel(
    const u32x4 *__restrict__ a, const u32x4 *__restrict__ b, uint64_t n_units, uint32_t units_per_block_log2,
    uint32_t *__restrict__ flags) {
  const uint32_t n_groups = (uint32_t)((n_units + 1023) / 1024), span = (n_groups + 7) / 8;
  const uint32_t g = (blockIdx.x & 7u) * span + (blockIdx.x >> 3);
  if (g >= n_groups) return;
  const uint64_t first = (uint64_t)g * 1024;
  const uint64_t left = n_units - first;
  const uint32_t mine = left < 1024 ? (uint32_t)left : 1024u;
  u32x4 x[4], y[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (threadIdx.x + 256u * i < mine) {
      x[i] = __builtin_nontemporal_load(a + first + threadIdx.x + 256 * i);
      y[i] = __builtin_nontemporal_load(b + first + threadIdx.x + 256 * i);
    }
  uint32_t diff = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (threadIdx.x + 256u * i < mine) {
      const u32x4 d = x[i] ^ y[i];
      diff |= d.x | d.y | d.z | d.w;
    }
  if (__ballot(diff != 0) != 0 && (threadIdx.x & (kWave - 1)) == 0) atomicOr(flags + (first >> units_per_block_log2), 1u);
}

// ---- block elision of an image (the compressed-snapshot experiment) ------------------------------------
// keep[k] = 1 if some 16-byte unit of block k differs from the block's first unit.  One work-group looks at
// 1024 units (16 KiB), which lie in one block (the block size is a power of two of at least 16 KiB).
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 4))) void ds_constant_blocks_kernel(
    const u32x4 *__restrict__ img, uint64_t n_units, uint32_t units_per_block_log2, uint32_t *__restrict__ keep) {
  const uint32_t n_groups = (uint32_t)((n_units + 1023) / 1024), span = (n_groups + 7) / 8;
  const uint32_t g = (blockIdx.x & 7u) * span + (blockIdx.x >> 3);
  if (g >= n_groups) return;
  const uint64_t first = (uint64_t)g * 1024;
  const uint64_t left = n_units - first;
  const uint32_t mine = left < 1024 ? (uint32_t)left : 1024u;
  const uint64_t block = first >> units_per_block_log2;
  const u32x4 ref = img[block << units_per_block_log2];
  u32x4 x[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (threadIdx.x + 256u * i < mine) x[i] = __builtin_nontemporal_load(img + first + threadIdx.x + 256 * i);
  uint32_t diff = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (threadIdx.x + 256u * i < mine) {
      const u32x4 d = x[i] ^ ref;
      diff |= d.x | d.y | d.z | d.w;
    }
  if (__ballot(diff != 0) != 0 && (threadIdx.x & (kWave - 1)) == 0) atomicOr(keep + block, 1u);
}

// pos[k] = keep[0] + ... + keep[k-1], pos[n] = the sum.  One work-group walks the array 256 entries at a time.
__global__ __launch_bounds__(256) void ds_exclusive_scan_kernel(const uint32_t *__restrict__ keep, uint32_t *__restrict__ pos,
                                                                 uint64_t n) {
  __shared__ uint32_t wave_sum[4];
  const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
  uint32_t carry = 0;
  for (uint64_t base = 0; base < n; base += 256) {
    const uint64_t i = base + tid;
    const uint32_t x = i < n ? keep[i] : 0u;
    const uint32_t incl = wave_inclusive_scan(x, lane);
    if (lane == kWave - 1) wave_sum[wv] = incl;
    __syncthreads();
    uint32_t before = carry;
    for (uint32_t w = 0; w < wv; ++w) before += wave_sum[w];
    if (i < n) pos[i] = before + incl - x;
    carry += wave_sum[0] + wave_sum[1] + wave_sum[2] + wave_sum[3];
    __syncthreads();
  }
  if (tid == 0) pos[n] = carry;
}

// Kept blocks go to their slots in `packed`, one behind the other; every block leaves its first unit in
// `patterns`.  Same work-group shape as above.
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 4))) void ds_pack_kept_blocks_kernel(
    const u32x4 *__restrict__ img, uint64_t n_units, uint32_t units_per_block_log2, const uint32_t *__restrict__ keep,
    const uint32_t *__restrict__ pos, u32x4 *__restrict__ patterns, u32x4 *__restrict__ packed) {
  const uint32_t n_groups = (uint32_t)((n_units + 1023) / 1024), span = (n_groups + 7) / 8;
  const uint32_t g = (blockIdx.x & 7u) * span + (blockIdx.x >> 3);
  if (g >= n_groups) return;
  const uint64_t first = (uint64_t)g * 1024;
  const uint64_t left = n_units - first;
  const uint32_t mine = left < 1024 ? (uint32_t)left : 1024u;
  const uint64_t block = first >> units_per_block_log2;
  const uint64_t in_block = first - (block << units_per_block_log2);
  if (in_block == 0 && threadIdx.x == 0) patterns[block] = img[first];
  if (!keep[block]) return;
  u32x4 *out = packed + ((uint64_t)pos[block] << units_per_block_log2) + in_block;
  u32x4 x[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (threadIdx.x + 256u * i < mine) x[i] = __builtin_nontemporal_load(img + first + threadIdx.x + 256 * i);
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (threadIdx.x + 256u * i < mine) __builtin_nontemporal_store(x[i], out + threadIdx.x + 256 * i);
}

}  // namespace

extern "C" int ds_image_compress(const void *image_dev, uint64_t nbytes, uint64_t block_bytes, uint32_t *keep_dev,
                                 uint32_t *pos_dev, void *patterns_dev, void *packed_dev, void *stream) {
  if (nbytes == 0) return DS_OK;
  if (!image_dev || !keep_dev || !pos_dev || !patterns_dev || !packed_dev ||
      (((uintptr_t)image_dev | (uintptr_t)patterns_dev | (uintptr_t)packed_dev) & 15) ||
      (((uintptr_t)keep_dev | (uintptr_t)pos_dev) & 3))
    return DS_EINVAL;
  // a power of two of at least 16 KiB, so that a work-group's piece lies in one block
  if (block_bytes < 16384 || (block_bytes & (block_bytes - 1)) || (nbytes & 15)) return DS_ERANGE;
  const uint64_t n_units = nbytes >> 4;
  const uint64_t groups = (n_units + 1023) / 1024;
  if (groups > 0x7FFFFFF0ull) return DS_ERANGE;
  const uint64_t n_blocks = (nbytes + block_bytes - 1) / block_bytes;
  const uint32_t upb_log2 = (uint32_t)__builtin_ctzll(block_bytes >> 4);
  const uint32_t grid = (uint32_t)(((groups + 7) / 8) * 8);
  hipStream_t st = (hipStream_t)stream;
  hipLaunchKernelGGL(ds_clear_flags_kernel, dim3((uint32_t)((n_blocks + 255) / 256)), dim3(256), 0, st, keep_dev, n_blocks);
  DS_HIP_TRY(hipGetLastError());
  hipLaunchKernelGGL(ds_constant_blocks_kernel, dim3(grid), dim3(256), 0, st, (const u32x4 *)image_dev, n_units, upb_log2,
                     keep_dev);
  DS_HIP_TRY(hipGetLastError());
  hipLaunchKernelGGL(ds_exclusive_scan_kernel, dim3(1), dim3(256), 0, st, keep_dev, pos_dev, n_blocks);
  DS_HIP_TRY(hipGetLastError());
  hipLaunchKernelGGL(ds_pack_kept_blocks_kernel, dim3(grid), dim3(256), 0, st, (const u32x4 *)image_dev, n_units, upb_log2,
                     keep_dev, pos_dev, (u32x4 *)patterns_dev, (u32x4 *)packed_dev);
  DS_HIP_TRY(hipGetLastError());
  return DS_OK;
}

extern "C" int ds_image_diff(const void *image_a_dev, const void *image_b_dev, uint64_t nbytes, uint64_t block_bytes,
                             uint32_t *changed_dev, void *stream) {
  if (nbytes == 0) return DS_OK;
  if (!image_a_dev || !image_b_dev || !changed_dev || (((uintptr_t)image_a_dev | (uintptr_t)image_b_dev) & 15) ||
      ((uintptr_t)changed_dev & 3))
    return DS_EINVAL;
  // a power of two of at least 16 KiB, so that a work-group's piece lies in one block
  if (block_bytes < 16384 || (block_bytes & (block_bytes - 1)) || (nbytes & 15)) return DS_ERANGE;
  const uint64_t n_units = nbytes >> 4;
  const uint64_t groups = (n_units + 1023) / 1024;
  if (groups > 0x7FFFFFF0ull) return DS_ERANGE;
  const uint64_t n_blocks = (nbytes + block_bytes - 1) / block_bytes;
  hipLaunchKernelGGL(ds_clear_flags_kernel, dim3((uint32_t)((n_blocks + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                     changed_dev, n_blocks);
  DS_HIP_TRY(hipGetLastError());
  const uint64_t grid = ((groups + 7) / 8) * 8;
  hipLaunchKernelGGL(ds_diff_kernel, dim3((uint32_t)grid), dim3(256), 0, (hipStream_t)stream, (const u32x4 *)image_a_dev,
                     (const u32x4 *)image_b_dev, n_units, (uint32_t)__builtin_ctzll(block_bytes >> 4), changed_dev);
  DS_HIP_TRY(hipGetLastError());
  return DS_OK;
}

extern "C" int ds_copy_probe(void *dst_dev, const void *src_dev, uint64_t nbytes, void *stream) {
  if (nbytes == 0) return DS_OK;
  if (!dst_dev || !src_dev || (((uintptr_t)dst_dev | (uintptr_t)src_dev | nbytes) & 15)) return DS_EINVAL;
  const uint64_t n_units = nbytes >> 4;
  const uint64_t groups = (n_units + 1023) / 1024;
  if (groups > 0x7FFFFFF0ull) return DS_ERANGE;
  const uint64_t grid = ((groups + 7) / 8) * 8;
  hipLaunchKernelGGL(ds_copy_probe_kernel, dim3((uint32_t)grid), dim3(256), 0, (hipStream_t)stream,
                     (const u32x4 *)src_dev, (u32x4 *)dst_dev, n_units);
  DS_HIP_TRY(hipGetLastError());
  return DS_OK;
}

namespace {

// The plan's tables in device memory: the plan's own copy, or the one ds_pack_noalloc keeps in static memory.
struct DeviceTables {
  const DsTile *tiles;
  const DsTileHot *hot;
  const uint32_t *first_tile;
  const DsChunkRec *recs;
};

int launch_move_with(const ds_plan *plan, const DeviceTables &tb, bool pack, uint8_t *img, uint64_t img_lo,
                     uint64_t img_hi, uint32_t grid_limit, hipStream_t stream) {
  const uint32_t lg = plan->chunk_log2;
  const uint64_t C = (uint64_t)1 << lg;
  const uint64_t n_total = plan->n_chunks();
  if (img_hi > plan->total_bytes || img_lo >= img_hi) return DS_ERANGE;
  // whole chunks inside the range: one work item each, lean or general by their record ...
  uint64_t w_lo = (img_lo + C - 1) >> lg;
  uint64_t w_hi = img_hi >> lg;
  if (img_hi == plan->total_bytes) w_hi = n_total;  // the last chunk may be short; its record says 'general' then
  LeanArgs la;
  la.recs = tb.recs;
  la.img = img;
  la.img_lo = img_lo;
  la.chunk_log2 = lg;
  la.c_lo = (uint32_t)w_lo;
  la.n_chunks = w_hi > w_lo ? (uint32_t)(w_hi - w_lo) : 0;
  la.xcd_span = ds_cfg_variant() == 3 ? 0 : (la.n_chunks + 7) / 8;
  // ... and the one or two chunks cut by the ends of the range, clipped by the general path
  MoveArgs ma;
  ma.tiles = tb.tiles;
  ma.hot = tb.hot;
  ma.first_tile = tb.first_tile;
  ma.img = img;
  ma.img_lo = img_lo;
  ma.img_hi = img_hi;
  ma.total = plan->total_bytes;
  ma.chunk_log2 = lg;
  ma.n_extra = 0;
  ma.extra[0] = ma.extra[1] = 0;
  const uint64_t c_first = img_lo >> lg, c_last = (img_hi - 1) >> lg;
  if (w_hi <= w_lo) {
    // no whole chunk: the range touches one or two chunks, both cut
    ma.extra[ma.n_extra++] = (uint32_t)c_first;
    if (c_last != c_first) ma.extra[ma.n_extra++] = (uint32_t)c_last;
  } else {
    if (c_first < w_lo) ma.extra[ma.n_extra++] = (uint32_t)c_first;
    if (c_last >= w_hi) ma.extra[ma.n_extra++] = (uint32_t)c_last;
  }
  const uint64_t variant = ds_cfg_variant();
  if (variant == 1) {  // plain loads and stores
    return pack ? launch_move<true, false, false, false>(lg, la, ma, grid_limit, stream)
                : launch_move<false, false, false, false>(lg, la, ma, grid_limit, stream);
  }
  if (variant == 2) {  // non-temporal global loads and stores everywhere (no buffer stores)
    return pack ? launch_move<true, true, true, false>(lg, la, ma, grid_limit, stream)
                : launch_move<false, true, true, false>(lg, la, ma, grid_limit, stream);
  }
  // default: non-temporal accesses, and the lean gather writes the image with "sc0 sc1 nt" buffer stores;
  // as many wavefronts per SIMD as the registers allow, up to six, instead of four where most of the plan's
  // chunks take the general path
  if (plan->n_general * 2 > n_total && variant != 5)
    return pack ? launch_move<true, true, true, true, 6>(lg, la, ma, grid_limit, stream)
                : launch_move<false, true, true, false, 6>(lg, la, ma, grid_limit, stream);
  return pack ? launch_move<true, true, true, true>(lg, la, ma, grid_limit, stream)
              : launch_move<false, true, true, false>(lg, la, ma, grid_limit, stream);
}

}  // namespace

int ds_launch_move(const ds_plan *plan, bool pack, uint8_t *img, uint64_t img_lo, uint64_t img_hi,
                   uint32_t grid_limit, hipStream_t stream) {
  // the tables live on the device the plan was made on: a launch from another one would read them remotely
  int dev = -1;
  DS_HIP_TRY(hipGetDevice(&dev));
  if (dev != plan->device) return DS_ESTATE;
  const DeviceTables tb = {plan->d_tiles, plan->d_hot, plan->d_first_tile, plan->d_recs};
  return launch_move_with(plan, tb, pack, img, img_lo, img_hi, grid_limit, stream);
}

// ---- ds_pack for callers that cannot allocate ----------------------------------------------------
// The gather reads the plan's tables from device memory; ds_plan_create puts them into an allocation of
// its own.  Here they go into a static device array instead, so that neither the plan (made with
// DS_PLAN_HOST_ONLY) nor the call allocates device memory.  Every device the library runs on holds its own
// copy of the array, at its own address, until the process ends.
namespace {

constexpr size_t kScratchBytes = DS_PACK_NOALLOC_TABLE_BYTES;
static __device__ __align__(256) uint8_t scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
uint8_t *g_scratch_ptr[kMaxDevices];  // device address of `scratch` on device d, once asked for

// The array's address on the current device (`dev`).  In host code the array's name is only a handle for
// this lookup, never an address a kernel or a copy could use.
int scratch_on_device(int dev, uint8_t **out) {
  if (dev < 0 || dev >= kMaxDevices) return DS_EINVAL;
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    DS_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return DS_EINVAL;
    g_scratch_ptr[dev] = (uint8_t *)p;
  }
  *out = g_scratch_ptr[dev];
  return DS_OK;
}

inline size_t round_up_128(size_t x) { return (x + 127) & ~(size_t)127; }

}  // namespace

extern "C" int ds_pack_noalloc(const ds_plan *plan, void *dst_dev, uint64_t img_lo, uint64_t img_hi, void *stream) {
  if (!plan) return DS_EINVAL;
  if (img_lo > img_hi || img_hi > plan->total_bytes || ((img_lo | img_hi) & 15)) return DS_ERANGE;
  // the tables, laid out one behind the other as in a plan's own device copy
  const size_t b_tiles = plan->tiles.size() * sizeof(DsTile);
  const size_t b_off = round_up_128(plan->hot.size() * sizeof(DsTileHot));
  const size_t b_first = round_up_128(plan->first_tile.size() * sizeof(uint32_t));
  const size_t b_recs = round_up_128(plan->recs.size() * sizeof(DsChunkRec));
  if (b_tiles + b_off + b_first + b_recs > kScratchBytes) return DS_ETOOBIG;
  if (img_lo == img_hi) return DS_OK;
  if (!dst_dev || ((uintptr_t)dst_dev & 15)) return DS_EINVAL;
  int dev = -1;
  DS_HIP_TRY(hipGetDevice(&dev));
  uint8_t *base = nullptr;
  const int rc = scratch_on_device(dev, &base);
  if (rc != DS_OK) return rc;
  // Copies and kernel on the caller's stream: they run behind whatever that stream still has to do with the
  // array (an earlier call's kernel).  Every entry the kernel reads is written here first, so nothing of an
  // earlier call's tables, which stay in the array, needs clearing.  The host tables belong to the plan, which
  // the caller keeps until the work has run.
  hipStream_t st = (hipStream_t)stream;
  if (b_tiles) DS_HIP_TRY(hipMemcpyAsync(base, plan->tiles.data(), b_tiles, hipMemcpyHostToDevice, st));
  DS_HIP_TRY(hipMemcpyAsync(base + b_tiles, plan->hot.data(), plan->hot.size() * sizeof(DsTileHot),
                            hipMemcpyHostToDevice, st));
  DS_HIP_TRY(hipMemcpyAsync(base + b_tiles + b_off, plan->first_tile.data(),
                            plan->first_tile.size() * sizeof(uint32_t), hipMemcpyHostToDevice, st));
  DS_HIP_TRY(hipMemcpyAsync(base + b_tiles + b_off + b_first, plan->recs.data(),
                            plan->recs.size() * sizeof(DsChunkRec), hipMemcpyHostToDevice, st));
  const DeviceTables tb = {(const DsTile *)base, (const DsTileHot *)(base + b_tiles),
                           (const uint32_t *)(base + b_tiles + b_off),
                           (const DsChunkRec *)(base + b_tiles + b_off + b_first)};
  return launch_move_with(plan, tb, true, (uint8_t *)dst_dev, img_lo, img_hi, 0, st);
}
