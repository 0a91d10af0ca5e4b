// Internal definitions shared by the host side and the kernels of
// libdatastates_hip.so.  Not part of the ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "datastates.h"

// A tile is one non-empty shard in device form: the view is normalised to
// "outer index -> start of a contiguous run of run_bytes".  Its place in the
// image is [tile_off[t], tile_off[t+1]): payload first, then padding.
struct DsTile {
  uint64_t src;        // device address of element (0,...,0)
  uint64_t nbytes;     // payload bytes
  uint64_t run_bytes;  // length of the innermost contiguous run; == nbytes when n_outer == 0
  uint32_t n_outer;    // outer dimensions left after merging; 0 = the whole shard is one run
  uint32_t es_log2;    // log2(itemsize)
  uint64_t extent[DS_MAX_DIMS];  // outer extents, slowest first
  uint64_t stride[DS_MAX_DIMS];  // outer strides in BYTES
};
static_assert(sizeof(DsTile) == 128, "DsTile is one 128-byte line");

// What the kernel's general path needs of a tile, 40 bytes instead of the 128 of a DsTile plus its two
// tile_off entries: the first wavefront of a general chunk reads one of these per lane.  Entry n_tiles is
// a sentinel whose img_off is the image length, so that a tile's end is the next entry's img_off.
struct DsTileHot {
  uint64_t img_off;  // where the tile's range starts in the image (= tile_off[t])
  uint64_t src;      // device address of element (0,...,0)
  uint64_t nbytes;   // payload bytes
  uint64_t stride0;  // distance between runs in bytes (views with one outer dimension)
  uint32_t run;      // run length in bytes, views with one outer dimension (0 otherwise)
  uint32_t meta;     // n_outer | log2(itemsize) << 8.  n_outer is given as 2 for a view with one outer
                     // dimension whose runs do not fit 32 bits: it then takes the routes of the N-D views
};
static_assert(sizeof(DsTileHot) == 40, "five 8-byte words");

// What the kernel's lean path needs to move one whole chunk, in one 32-byte load.
// Chunks that are not "simple" (a tile boundary, the end of a payload or
// padding inside the chunk, more than one outer dimension, rows shorter than
// 16 bytes) are of kind DS_CHUNK_GENERAL and take the general path; their
// record names the tiles they hold (tile, col0).
enum : uint32_t { DS_CHUNK_CONTIG = 0, DS_CHUNK_ROWS = 1, DS_CHUNK_GENERAL = 2 };
// CONTIG only, bit 8 of `kind`: the tensor side of the chunk is not 16-byte aligned, and the tensor has at least
// 16 more bytes on either side of it, so the gather may read the 16-byte aligned units that cover the chunk's
// bytes (one more than the chunk has) without leaving the tensor.
enum : uint32_t { DS_CHUNK_REALIGN = 1u << 8 };
struct DsChunkRec {
  uint64_t addr;   // CONTIG: tensor address of the chunk's first byte; ROWS: address of the run that holds it
  uint64_t pitch;  // ROWS: distance between runs in bytes
  uint32_t col0;   // ROWS: position of the chunk's first byte inside its run.  GENERAL: number of tiles after the first
  uint32_t run;    // ROWS: run length in bytes (>= 16, multiple of the itemsize)
  uint32_t kind;   // low byte: DS_CHUNK_*; bits 8..: log2(itemsize) (ROWS), DS_CHUNK_REALIGN (CONTIG)
  uint32_t tile;   // GENERAL: first tile of the chunk.  ROWS: (step / run) << 16 | (step % run), step = bytes
                   // between two units of one thread (threads per work-group x 16)
};
static_assert(sizeof(DsChunkRec) == 32, "two records per 64 bytes");

struct DsManifestEntry {
  uint64_t tensor_id;
  uint32_t dtype;
  uint32_t ndim;
  int64_t shape[DS_MAX_DIMS];  // unused extents 0
  uint64_t file_offset;   // inside the shard's own file
  uint64_t nbytes;
  uint64_t image_offset;  // in the plan's image (= file_offset + where the file's region starts)
  uint32_t file;
};

// One file of a flush or of a restore: image bytes [begin, end) are the file's bytes [0, end - begin).
// fd_direct may be -1.
struct DsFileTarget {
  uint64_t begin = 0, end = 0;
  int fd_buffered = -1, fd_direct = -1;
};

// The flush of a snapshot into a file that somebody else opened and will close (the checkpoint writer).
// fd_direct may be -1.
int ds_flush_start_fds(ds_event *ev, int fd_buffered, int fd_direct, uint32_t threads, uint32_t flags, ds_flush **out);
// The same into several files: the targets are in image order, the first begins at 0 and each begins where
// the one before ends.  May throw std::bad_alloc (the vector is taken by value).
int ds_flush_start_targets(ds_event *ev, std::vector<DsFileTarget> targets, uint32_t threads, uint32_t flags,
                           ds_flush **out);
// Image -> tensors out of files that the caller opened and will close; the targets must cover the image.
int ds_restore_from_targets(ds_engine *engine, const ds_plan *plan, const std::vector<DsFileTarget> &targets,
                            uint32_t threads, void *compute_stream, ds_event **out);
const ds_plan *ds_event_plan(const ds_event *ev);  // the plan a snapshot or restore was started with
void ds_set_errno(int e);  // what ds_last_errno() returns on this thread
bool ds_io_uring_available();  // can this process set up an io_uring?
void ds_drop_pinned_cache();   // frees the pinned ring kept from a destroyed engine

struct ds_plan {
  uint64_t align = 0;
  uint64_t total_bytes = 0;
  uint64_t payload_bytes = 0;
  uint64_t n_shards = 0;
  uint64_t n_strided = 0;
  uint32_t chunk_log2 = 0;
  std::vector<DsManifestEntry> manifest;   // table order as given
  std::vector<uint64_t> file_begin;        // n_files + 1 entries: where each file's tensor region starts in the image
  std::vector<DsTile> tiles;               // image order
  std::vector<uint64_t> tile_off;          // n_tiles + 1 entries, last = total_bytes (host only)
  std::vector<DsTileHot> hot;              // n_tiles + 1 entries, image order, last = sentinel
  std::vector<uint32_t> first_tile;        // n_chunks + 1 entries, last = n_tiles
  std::vector<DsChunkRec> recs;            // one per chunk
  uint64_t n_general = 0;                  // chunks of kind DS_CHUNK_GENERAL
  // device copies (one allocation)
  int device = -1;
  void *dev_blob = nullptr;
  const DsTile *d_tiles = nullptr;
  const DsTileHot *d_hot = nullptr;
  const uint32_t *d_first_tile = nullptr;
  const DsChunkRec *d_recs = nullptr;
  uint64_t n_chunks() const { return first_tile.empty() ? 0 : first_tile.size() - 1; }
};

// ---- error plumbing ---------------------------------------------------------
void ds_set_hip_error(hipError_t e);
#define DS_HIP_TRY(expr)                 \
  do {                                   \
    hipError_t _e = (expr);              \
    if (_e != hipSuccess) {              \
      ds_set_hip_error(_e);              \
      return DS_EHIP;                    \
    }                                    \
  } while (0)

// ---- tunables ---------------------------------------------------------------
uint64_t ds_cfg_chunk_bytes();
uint64_t ds_cfg_variant();

// ---- kernel launchers (ds_kernels.hip) ---------------------------------------
// Moves image bytes [img_lo, img_hi) between the tensors of `plan` and `img`
// (which points at image byte img_lo).  pack: tensors -> img; else img -> tensors.
// grid_limit 0 = one work-group per chunk.
int ds_launch_move(const ds_plan *plan, bool pack, uint8_t *img, uint64_t img_lo, uint64_t img_hi,
                   uint32_t grid_limit, hipStream_t stream);
