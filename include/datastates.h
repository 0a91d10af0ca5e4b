/*
 * datastates.h -- C ABI of the MI355X snapshot hot path (libdatastates_hip.so).
 *
 * One GPU's part of the lazy, non-blocking checkpoint snapshot of
 * DataStates-LLM (arXiv 2601.16956): the fragmented, mixed-precision, possibly
 * strided model/optimizer shards of one rank are coalesced into one contiguous
 * image laid out like the checkpoint file (Sec. V-A1 "coalescing", Sec. V-A5
 * rule (1): offsets fixed in advance), the image is streamed to a pre-pinned,
 * reused host ring (Sec. V-A1; the circular host cache of Sec. V-B/V-C) in chunks that
 * need not be whole tensors (Sec. V-A4), while training continues; the
 * mutating update phase is gated on the capture (Sec. V-A2).  Restore is the
 * inverse scatter.
 *
 * Conventions
 *   - Plain C.  No HIP or torch types: a stream is passed as `void*` holding a
 *     hipStream_t (NULL = the null stream).  "dev" pointers are device
 *     addresses valid on the device that was current when the plan / engine
 *     was created; "host" pointers are ordinary host addresses.
 *   - Every function returns an int: DS_OK (0), a positive status
 *     (DS_NOT_READY, DS_EOF) or a negative error.  Nothing throws or aborts.
 *     Out-parameters are written only on DS_OK (or the documented status).
 *   - A plan is immutable once created and may be used from several threads.
 *     Requests on one engine (create / destroy, ds_snapshot_async,
 *     ds_restore_*) are serialised by the caller; the calls on an event may
 *     come from other threads than the request -- the gate from the training
 *     thread, ds_snapshot_next_chunk from ONE consumer thread, and
 *     ds_snapshot_release_chunk from any number of threads (a flush does
 *     exactly that).
 *   - The image.  For shard i:  bytes_i = itemsize(dtype_i) * prod(shape_i)
 *     (empty product = 1).  Image byte  file_offset_i + r*itemsize + b  is byte
 *     b of the element of rank r in the row-major (last index fastest)
 *     enumeration of the VIEW, which lives at
 *     base_i + itemsize * sum_j k_j * strides_i[j].  Bytes as they are: no
 *     dtype conversion, no byte swap (Sec. IV-D, Sec. V-A3: tensors are
 *     byte-addressable buffers that need no serialisation).  Every image byte
 *     that belongs to no shard is 0x00.  The image length is the end of the
 *     last shard rounded up to the alignment.
 */
#ifndef DATASTATES_H
#define DATASTATES_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DS_MAX_DIMS 6

/* element types; only the size matters to the byte mover: 4, 2, 2, 8, 1 */
typedef enum ds_dtype { DS_F32 = 0, DS_BF16 = 1, DS_F16 = 2, DS_I64 = 3, DS_U8 = 4 } ds_dtype;

/* status and error codes */
#define DS_OK 0
#define DS_NOT_READY 1 /* ds_event_query: snapshot still in flight               */
#define DS_EOF 2       /* ds_snapshot_next_chunk: every chunk has been handed out */
#define DS_EINVAL (-1)   /* null pointer, bad dtype/ndim/shape/stride/alignment value, misaligned base */
#define DS_EALIGN (-2)   /* a file_offset is not a multiple of the alignment      */
#define DS_EOVERLAP (-3) /* two shards intersect in the image, or a view addresses an element twice */
#define DS_EGAP (-4)     /* DS_PLAN_STRICT: a hole that is not alignment padding  */
#define DS_ERANGE (-5)   /* image range outside [0,total], reversed, or not a multiple of 16 */
#define DS_ENOMEM (-6)   /* host or device allocation failed                      */
#define DS_EHIP (-7)     /* a HIP call failed; see ds_last_hip_error()            */
#define DS_EBUSY (-8)    /* object still has work in flight / chunk not released  */
#define DS_ESTATE (-9)   /* call not valid in this state (e.g. release of a chunk never handed out) */
#define DS_EIO (-10)     /* a file operation failed; see ds_last_errno()           */
#define DS_EFORMAT (-11) /* not a checkpoint file of this format, or a damaged one   */
#define DS_EFAULT (-12)  /* DS_PLAN_CHECK_MEMORY: a shard is not inside one device allocation */
#define DS_ETOOBIG (-13) /* ds_pack_noalloc: the plan's tables do not fit the static table memory */

/*
 * One shard: a view into device memory plus its place in the file.
 * (Sec. IV-C: a rank owns many separate shards, cut where the parallel
 * execution plan and the optimizer sharding put the cuts, not where a
 * checkpoint layout would.)
 */
typedef struct ds_shard_desc {
  const void *base;               /* DEVICE address of element (0,...,0); multiple of the itemsize */
  uint32_t dtype;                 /* ds_dtype                                                     */
  uint32_t ndim;                  /* 0..DS_MAX_DIMS; 0 = exactly one element                      */
  int64_t shape[DS_MAX_DIMS];     /* extents >= 0 (a zero extent = empty shard, 0 bytes)          */
  int64_t strides[DS_MAX_DIMS];   /* in ELEMENTS, > 0 for every extent > 1; the view must not
                                     address any element twice (DS_EOVERLAP).  Checked exactly:
                                     by the nesting of the strides where they nest (any slice,
                                     transpose or permutation of a dense parent does), else by
                                     writing out the addresses, which is done for views of up
                                     to 2^20 elements; a larger view with strides that do not
                                     nest is refused                                              */
  uint64_t tensor_id;             /* logical tensor this shard is a slice of; kept in the plan's
                                     manifest, never touches the bytes                            */
  uint64_t file_offset;           /* byte offset of the shard in the image; multiple of `align`   */
} ds_shard_desc;

typedef struct ds_plan ds_plan;
typedef struct ds_engine ds_engine;
typedef struct ds_event ds_event;
typedef struct ds_flush ds_flush;
typedef struct ds_ckpt ds_ckpt;               /* a checkpoint file being written */
typedef struct ds_ckpt_reader ds_ckpt_reader; /* a checkpoint file opened for recovery */

/* ---- layout and plan (Sec. V-A3 composite provider, duty (a): sizes and
 *      offsets in the stream; Sec. V-A5 rule (1)) ---------------------------- */

/* Size of one element in bytes, 0 for an unknown dtype. */
int ds_itemsize(uint32_t dtype);

/*
 * Canonical layout: writes file_offset of desc[0..n) in table order, each at
 * the next multiple of `align` after the end of the one before; *total = image
 * length (a multiple of `align`).  Host-only, touches no device.
 * `align` must be a power of two >= 16.  Errors: DS_EINVAL.
 */
int ds_layout_assign(ds_shard_desc *desc, size_t n, uint64_t align, uint64_t *total);

#define DS_PLAN_STRICT 1u    /* reject holes larger than alignment padding (DS_EGAP)           */
#define DS_PLAN_HOST_ONLY 2u /* validate and build tables on the host only; such a plan can be
                                inspected but not passed to ds_pack/ds_unpack/ds_snapshot_async */
#define DS_PLAN_CHECK_MEMORY 4u /* ask the runtime, for every non-empty shard, which allocation its
                                base address lies in, and require every address of the view to be
                                inside it (DS_EFAULT otherwise): a wrong descriptor is then an error
                                here, not a memory fault in a kernel later.  Costs one runtime call
                                per shard; not with DS_PLAN_HOST_ONLY */

/*
 * Validates the table (any order of offsets; shards must be disjoint in the
 * image), normalises every view (merges dimensions that are contiguous with
 * each other, splits off the innermost contiguous run), cuts the image into
 * work-group chunks and uploads the tables to the current device.  The
 * descriptors are copied: the caller may free `desc` afterwards.  The tensors
 * themselves stay owned by the caller and must stay allocated while the plan
 * is used.  The plan is reused by every snapshot of the same shard set (Sec.
 * V-A1: what is set up once serves all later checkpoint requests).
 * Errors: DS_EINVAL, DS_EALIGN, DS_EOVERLAP, DS_EGAP, DS_EFAULT, DS_ENOMEM, DS_EHIP.
 */
int ds_plan_create(const ds_shard_desc *desc, size_t n, uint64_t align, uint32_t flags, ds_plan **out);

/*
 * One plan for a rank that writes its checkpoint as several files (Sec. VI-D:
 * 20 files for a 7B rank; Sec. V-A3: one composite provider per rank lays out
 * everything it owns).  file_of[i] < n_files names the file of shard i and
 * desc[i].file_offset counts from the start of THAT file.  The plan's one image
 * is the files' tensor regions one behind the other in file order: region f
 * spans the shards of file f from offset 0 up to the end of the last one,
 * rounded up to `align`, and starts at the sum of the regions before it (see
 * ds_plan_file).  One gather launch and one snapshot then cover all files, and
 * the file tier cuts the image at the region boundaries (ds_flush_start_files,
 * ds_ckpt_flush_snapshot_parts).  A file that no shard names has an empty
 * region.  file_of == NULL with n_files == 1 is ds_plan_create.  Everything else
 * (checks, flags, errors, ownership) as ds_plan_create; DS_PLAN_STRICT also
 * requires every file's first shard at offset 0.  n_files <= DS_MAX_FILES.
 */
#define DS_MAX_FILES 65536u
int ds_plan_create_files(const ds_shard_desc *desc, const uint32_t *file_of, size_t n, uint32_t n_files,
                         uint64_t align, uint32_t flags, ds_plan **out);

/* ds_layout_assign file by file: the canonical offset of every shard inside its own
 * file; region_bytes[n_files] (may be NULL) gets the files' tensor-region lengths,
 * *total their sum = the length of the image of ds_plan_create_files.
 * Errors: DS_EINVAL. */
int ds_layout_assign_files(ds_shard_desc *desc, const uint32_t *file_of, size_t n, uint32_t n_files,
                           uint64_t align, uint64_t *region_bytes, uint64_t *total);

/* Frees host and device tables.  The caller makes sure no kernel that uses
 * the plan is still running (synchronise the streams it was used on). */
int ds_plan_destroy(ds_plan *plan);

typedef struct ds_plan_stats {
  uint64_t total_bytes;   /* image length T                                       */
  uint64_t payload_bytes; /* sum of bytes_i; T - payload = padding                */
  uint64_t n_shards;      /* descriptors given                                    */
  uint64_t n_tiles;       /* non-empty shards (+1 if the image starts with a hole)*/
  uint64_t n_chunks;      /* work-group chunks over the whole image               */
  uint64_t chunk_bytes;   /* image bytes per work-group chunk                     */
  uint64_t n_strided;     /* shards that are not one contiguous run               */
  uint64_t align;
  uint64_t n_general_chunks; /* chunks that take the kernel's general path (the lean path takes the rest) */
  uint64_t n_files;       /* 1 for a plan of ds_plan_create                       */
} ds_plan_stats;

int ds_plan_info(const ds_plan *plan, ds_plan_stats *out);

/* Manifest entry i (table order as given): what a file header would record
 * (Sec. V-A5 rule (3)).  Any out pointer may be NULL. */
int ds_plan_shard(const ds_plan *plan, size_t i, uint64_t *tensor_id, uint32_t *dtype,
                  uint64_t *file_offset, uint64_t *nbytes);

/* File f of the plan: where its tensor region starts in the image and how long
 * it is.  Either out pointer may be NULL.  Errors: DS_EINVAL (f >= n_files). */
int ds_plan_file(const ds_plan *plan, uint32_t f, uint64_t *image_begin, uint64_t *region_bytes);

/* Manifest entry i: the file it belongs to and its offset in the IMAGE
 * (= the file_offset of ds_plan_shard + the file's image_begin). */
int ds_plan_shard_file(const ds_plan *plan, size_t i, uint32_t *file, uint64_t *image_offset);

/* Shape of manifest entry i: *ndim and the first *ndim extents of shape[DS_MAX_DIMS]
 * (the rest are set to 0).  Either out pointer may be NULL. */
int ds_plan_shard_shape(const ds_plan *plan, size_t i, uint32_t *ndim, int64_t *shape);

/* ---- the kernels (gather = Sec. V-A1 coalescing done on the device; scatter
 *      = recovery, Sec. V-A5 rule (3)) -------------------------------------- */

/*
 * Gather: writes image bytes [img_lo, img_hi) to dst_dev[0 .. img_hi-img_lo),
 * i.e. dst_dev points at where image byte img_lo goes (a staging slot, or the
 * start of a full-size buffer with img_lo = 0).  Padding bytes are written as
 * zero, so the destination need not be cleared.  img_lo <= img_hi <= total,
 * both multiples of 16; dst_dev 16-byte aligned.  Asynchronous: enqueued on
 * `stream`; the tensors must not change until it has run.  The device the
 * plan was created on must be the calling thread's current device (DS_ESTATE).
 * Errors: DS_EINVAL, DS_ERANGE, DS_ESTATE, DS_EHIP.
 */
int ds_pack(const ds_plan *plan, void *dst_dev, uint64_t img_lo, uint64_t img_hi, void *stream);

/*
 * Scatter, the exact inverse: every addressed element of every shard whose
 * image bytes lie in [img_lo, img_hi) is overwritten with src_dev[offset -
 * img_lo ...]; elements are written whole only if all their bytes are in the
 * range (ranges are multiples of 16 and itemsizes divide 16, so an element is
 * never cut).  No other byte of the tensors' memory is written.
 */
int ds_unpack(const ds_plan *plan, const void *src_dev, uint64_t img_lo, uint64_t img_hi, void *stream);

/*
 * ds_pack for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same result
 * as ds_pack, byte for byte; the difference is where the kernel finds the
 * plan's tables.  ds_pack reads them from the device allocation ds_plan_create
 * made; this call copies them (on `stream`, ahead of the kernel) into a static
 * device array of DS_PACK_NOALLOC_TABLE_BYTES that the library holds on every
 * GPU it runs on until the process ends, and calls neither hipMalloc nor
 * hipFree nor anything else that allocates.  `plan` may therefore be a
 * DS_PLAN_HOST_ONLY plan, whose creation touches no device either.
 * Limit: the tables (168 bytes per non-empty shard, 36 bytes per work-group
 * chunk of the image, i.e. about 2.3 KiB per MiB of image) must fit the array:
 * an image of about 1.7 GB with few shards does, DS_ETOOBIG otherwise
 * (returned before anything is enqueued).  All calls on one GPU share the one
 * array and it keeps the last call's tables: calls on the same stream are
 * ordered by it, calls that may overlap on one GPU (different streams, or
 * different threads) race and are the caller's to serialise.  Arguments and
 * the other errors as for ds_pack; the current device is the one that runs it.
 */
#define DS_PACK_NOALLOC_TABLE_BYTES (4u << 20)
int ds_pack_noalloc(const ds_plan *plan, void *dst_dev, uint64_t img_lo, uint64_t img_hi, void *stream);

/* ---- the snapshot engine (Sec. V-A1 pre-pinned reused pool, Sec. V-A2 lazy
 *      capture, Sec. V-A4 chunked streaming, Sec. V-C dedicated streams) ----- */

#define DS_ENGINE_AUTO_RELEASE 1u /* no consumer: a ring slot is reusable as soon as its copy is done */
#define DS_ENGINE_TRACE 2u        /* time every device-to-host copy of a snapshot (two events per chunk), for
                                     ds_event_trace */

typedef struct ds_engine_opts {
  uint64_t host_ring_bytes;  /* pinned host ring capacity, allocated and pinned once; the paper's
                                single tunable (Sec. V-B).  0 = 2 GiB                              */
  uint64_t d2h_chunk_bytes;  /* size of one ring slot = one device-to-host copy; multiple of 4096.
                                0 = 128 MiB (on one copy stream the gap between two copies costs
                                4 % of the link at 32 MiB, 1 % at 128 MiB)                          */
  uint64_t stage_slot_bytes; /* image bytes per gather launch (the last launch of an image may be
                                shorter); multiple of d2h_chunk_bytes.  0 = 1 GiB                   */
  uint32_t stage_slots;      /* device staging is one ring of stage_slots * stage_slot_bytes bytes
                                (>= 1; 0 = 2): a launch takes the next piece of it, of its own length,
                                so queued snapshots of small images share it.  With staging as large
                                as everything requested at a time, every gate opens after the gathers
                                alone, whatever the link, the host ring or the storage are doing    */
  uint32_t pack_grid_limit;  /* max work-groups resident per gather launch; 0 = one per chunk       */
  uint32_t flags;            /* DS_ENGINE_*                                                         */
  uint32_t copy_streams;     /* copy streams the chunks alternate over: 1 or 2.  0 = 1.  With 2 the gap
                                between two copies on one stream is hidden by the other stream's copy
                                (+2 % at 32 MiB chunks) -- when the two copies share the link evenly;
                                measured, they do in the first engine of a process and share it 2:1 in
                                later ones (-17 %), so one stream with large chunks is the default     */
  uint64_t first_launch_bytes; /* image bytes of the first gather launch of a snapshot; multiple of
                                d2h_chunk_bytes, <= stage_slot_bytes.  A short first launch lets the
                                first copy start earlier; the gather of the rest then runs beside that
                                copy.  0 = stage_slot_bytes (no short first launch)                  */
} ds_engine_opts;

/* Allocates the pinned ring, the device staging, a gather stream and the copy streams
 * (all at the default priority) and a host thread that issues the work.
 * Uses the current device.  The pinned ring and the device staging of a
 * destroyed engine are kept (one allocation each per process, the largest seen)
 * and handed to the next engine that fits into them: pinning is slow, a fresh
 * allocation is slow on first touch, and the first pinned allocation of a
 * process was measured to be the one the link writes fastest; the engine's
 * streams are reused likewise.  ds_config_set("drop_pinned_cache", 1) frees the
 * memory.
 * Errors: DS_EINVAL, DS_ENOMEM, DS_EHIP. */
int ds_engine_create(const ds_engine_opts *opts, ds_engine **out);

/* Waits for all snapshots in flight, then frees everything.  Events created
 * from the engine must have been destroyed.  Errors: DS_EBUSY, DS_EHIP. */
int ds_engine_destroy(ds_engine *engine);

/*
 * Checkpoint request (Sec. V-A2): records the point of consistency on
 * `compute_stream` and returns at once; gather launches and device-to-host
 * copies are issued by the engine's thread on its own streams and overlap
 * with whatever the caller enqueues next.  Between this call and the gate
 * (ds_event_wait_on_stream / ds_event_wait_captured) the caller must not
 * enqueue work that writes the tensors.  Snapshots on one engine run in the
 * order requested.  *out is owned by the caller (ds_event_destroy).
 * DS_EBUSY while a restore event of the engine is alive.
 */
int ds_snapshot_async(ds_engine *engine, const ds_plan *plan, void *compute_stream, ds_event **out);

/*
 * The lazy gate (Sec. V-A2: the update phase is delayed only if the copies
 * have not finished): makes `stream` wait until every source byte has been
 * read into staging.  Returns when the wait has been enqueued; blocks the
 * host only while the engine has not yet issued the last gather (e.g. the
 * host ring is full and the consumer is behind: the paper's back-pressure).
 * Hence, when staging is smaller than the images requested and not yet
 * copied out, the thread that calls the gate must not be the one that
 * consumes the chunks: it would wait for room that only it can make.
 */
int ds_event_wait_on_stream(ds_event *ev, void *stream);

/* Host-side form of the gate: returns when every source byte has been read. */
int ds_event_wait_captured(ds_event *ev);

/* DS_OK when the whole image has reached the host ring, else DS_NOT_READY. */
int ds_event_query(ds_event *ev);

/* Blocks the host until the whole image has reached the host ring (with a
 * consumer: until the last chunk's copy is done, which needs ring slots). */
int ds_event_wait(ds_event *ev);

/*
 * Consumer side (Sec. V-A3: the stream is exposed chunk by chunk, each an
 * address and a length): blocks until the next chunk of the image is resident in the ring,
 * then returns its host address, its offset in the image (which is the offset in
 * the file for a plan of one file; ds_plan_file maps it for a plan of several)
 * and its length.  Chunks come in image order.  DS_EOF after the last.  The memory stays valid
 * until ds_snapshot_release_chunk.  Not used with DS_ENGINE_AUTO_RELEASE.
 */
int ds_snapshot_next_chunk(ds_event *ev, const void **host_ptr, uint64_t *file_off, uint64_t *len);

/* Gives the ring slot back (Sec. V-A2: eviction after flush lets the next
 * request proceed).  Errors: DS_ESTATE if host_ptr is not a chunk handed out. */
int ds_snapshot_release_chunk(ds_event *ev, const void *host_ptr);

typedef struct ds_snapshot_stats {
  uint64_t image_bytes;
  uint64_t payload_bytes;
  uint32_t n_pack_launches;
  uint32_t n_copies;
  double pack_ms;       /* sum of gather kernel durations (HIP events on the gather stream)   */
  double copy_ms;       /* sum of device-to-host copy durations (HIP events on the copy stream) */
  double capture_ms;    /* request -> last source byte read                                   */
  double total_ms;      /* request -> last byte in the host ring                              */
  double submit_host_ms;/* host time spent inside ds_snapshot_async                           */
} ds_snapshot_stats;

/* Valid after ds_event_wait returned DS_OK. */
int ds_event_stats(ds_event *ev, ds_snapshot_stats *out);

/* One step of a snapshot on the device's clock, in milliseconds since the request
 * (what Sec. VI-D's timeline of tensors across the tiers shows, for this pipeline). */
typedef struct ds_trace_rec {
  uint32_t kind;      /* 0 = gather launch, 1 = device-to-host copy of one chunk */
  uint32_t index;     /* launch number / chunk number                           */
  uint64_t file_off;  /* image range the step covers                            */
  uint64_t len;
  double begin_ms;
  double end_ms;
} ds_trace_rec;

/*
 * Writes the records of a finished snapshot to out[0 .. cap): the gather
 * launches, then -- on an engine with DS_ENGINE_TRACE -- the copies in chunk
 * order.  *n = number of records there are (call with cap = 0 to ask).
 * Errors: DS_EBUSY (not finished), DS_ESTATE (a restore event), DS_EHIP.
 */
int ds_event_trace(ds_event *ev, ds_trace_rec *out, size_t cap, size_t *n);

/* Waits for the snapshot, releases chunks still held, frees the event. */
int ds_event_destroy(ds_event *ev);

/* ---- restore from a host image (recovery, Sec. V-A5 rule (3); the mirror image
 *      of the snapshot pipeline: pinned ring -> device staging -> scatter) ------ */

/*
 * Starts a restore of the whole image of `plan` through the engine's ring and
 * staging.  The engine must be idle: no snapshot or restore event of it may be
 * alive (DS_EBUSY).  Scatters are ordered after everything enqueued so far on
 * `compute_stream`.  The caller then repeats, in file order:
 *   ds_restore_next_slot  -> a ring slot to fill with image bytes
 *                            [file_off, file_off+len) (e.g. read from the file)
 *   ds_restore_submit     -> the slot is copied to the device; every eight chunks
 *                            (or stage_slot_bytes, if that is less) are scattered
 *                            into the tensors while the next ones are copied
 * and finally ds_event_wait (host) or ds_event_wait_on_stream (a stream that is
 * to use the restored tensors), then ds_event_destroy.
 */
int ds_restore_begin(ds_engine *engine, const ds_plan *plan, void *compute_stream, ds_event **out);

/*
 * Next ring slot, in file order.  Blocks the host only while the copy that last
 * used the slot is still in flight.  Several slots may be held at once (to read
 * ahead); DS_EBUSY if all of them are with the caller; DS_EOF after the last.
 */
int ds_restore_next_slot(ds_event *ev, void **host_ptr, uint64_t *file_off, uint64_t *len);

/* The slot has been filled.  Slots are submitted in the order they were handed
 * out (DS_ESTATE otherwise).  Returns as soon as the work is enqueued. */
int ds_restore_submit(ds_event *ev, const void *host_ptr);

/* ---- host <-> file tier (Sec. V-A4: a chunk goes on to the next tier as soon
 *      as it is resident; Sec. V-C: persistence on background threads) -------- */

#define DS_FILE_DIRECT 1u /* O_DIRECT for every transfer whose offset and length are multiples of 4 KiB
                             (ring slots are): straight from / into the ring where the kernel can pin the
                             ring's pages, else through an aligned buffer of ordinary memory (one extra
                             memory-speed copy, no page cache); anything else, and everything on a file
                             system without direct I/O, goes through a buffered descriptor */
#define DS_FILE_URING 4u  /* writes of a flush go through the kernel's io_uring interface: one thread keeps up
                             to `threads` writes in flight (Sec. V-C); where the process may not have an
                             io_uring (ds_config_get("io_uring_available") = 0) the pwrite threads are used */
#define DS_FILE_SYNC 2u   /* fsync before ds_flush_wait returns                                        */

/*
 * Starts the consumer of a snapshot taken on an engine WITHOUT
 * DS_ENGINE_AUTO_RELEASE: one thread takes the chunks as they land in the ring,
 * `threads` writer threads (0 = 4, at most 64) write each at its file offset
 * into `path` (created / truncated) and give the ring slot back.  Returns at
 * once.  The caller must not call ds_snapshot_next_chunk on `ev` itself.
 * Errors: DS_EINVAL, DS_ENOMEM, DS_EIO.
 */
int ds_flush_start(ds_event *ev, const char *path, uint32_t threads, uint32_t flags, ds_flush **out);

/*
 * The same for a snapshot of a plan of several files (ds_plan_create_files):
 * paths[f] gets the bytes of region f at file offsets 0.., so that file f is
 * exactly what ds_flush_start would write for a plan of file f's shards alone.
 * One set of `threads` writers serves all files; a ring chunk that spans a
 * region boundary is written in pieces and its slot is given back when the
 * last piece is out.  n_files must be the plan's.  Errors: as ds_flush_start.
 */
int ds_flush_start_files(ds_event *ev, const char *const *paths, uint32_t n_files, uint32_t threads,
                         uint32_t flags, ds_flush **out);

/* Waits until the whole image is in the file, closes it and frees the flush.
 * Either out pointer may be NULL.  Errors: DS_EIO (ds_last_errno()), or the
 * error that ended the snapshot. */
int ds_flush_wait(ds_flush *flush, uint64_t *bytes_written, double *seconds);

/*
 * Restore from a file written by a flush: reads the image with `threads`
 * reader threads into ring slots and feeds the restore pipeline
 * (ds_restore_begin / next_slot / submit) in file order.  Returns when the last
 * chunk has been submitted; *out is then waited for and destroyed like any
 * restore event.  The engine must be idle.  Errors: as ds_restore_begin, DS_EIO.
 */
int ds_restore_from_file(ds_engine *engine, const ds_plan *plan, const char *path, uint32_t threads,
                         uint32_t flags, void *compute_stream, ds_event **out);

/* The same out of the n_files files of a plan of several files, paths[f]
 * holding region f from its offset 0: ONE restore event, one scatter pipeline
 * for the whole rank.  n_files must be the plan's.  Errors: as above. */
int ds_restore_from_files(ds_engine *engine, const ds_plan *plan, const char *const *paths, uint32_t n_files,
                          uint32_t threads, uint32_t flags, void *compute_stream, ds_event **out);

/* errno of the file operation that last produced DS_EIO on this thread. */
int ds_last_errno(void);

/* ---- the checkpoint file (Sec. V-A5: tensors at offsets fixed in advance,
 *      serialized objects appended behind them as a concurrent log, a metadata
 *      header at the END of the file that describes both) ---------------------
 *
 * Layout, all integers little-endian:
 *   [0, T)            the tensor region: the image of the plan, byte for byte
 *   [T, E)            the object log.  A chunk of len bytes claims the next
 *                     round_up(len, 8) bytes; bytes never written read as 0
 *   [E, E+80n+32m)    the trailer: n tensor entries, then m chunk entries
 *       tensor entry (80 B): u64 tensor_id, u32 dtype, u32 ndim, u64 shape[6]
 *                     (unused extents 0), u64 file_offset, u64 nbytes; plan order
 *       chunk entry (32 B): u64 object_id, u64 seq, u64 file_offset, u64 len;
 *                     sorted by (object_id, seq); an object is the concatenation
 *                     of its chunks seq = 0, 1, ...
 *   last 64 B         the footer: char magic[8] = "DSCKPT01", u32 version = 1,
 *                     u32 flags = 0, u64 align, u64 T, u64 E, u64 n, u64 m,
 *                     u32 crc of the trailer, u32 crc of the 60 footer bytes before
 *                     it (CRC-32 of IEEE 802.3, as in zlib)
 * The paper fixes the three rules, not the bytes: the encoding is this library's.
 * A rank that writes several files per checkpoint uses either one plan and one
 * ds_ckpt per file, or ONE plan of several files (ds_plan_create_files) with one
 * ds_ckpt per file made by ds_ckpt_create_part: file f then holds region f of
 * the image as its tensor region, the plan's entries of file f (offsets inside
 * the file) as its tensor entries and an object log of its own -- byte for byte
 * the file that a plan of file f's shards alone would give.
 */

/*
 * Creates / truncates `path` for a checkpoint of `plan` (which may be a
 * DS_PLAN_HOST_ONLY plan when the tensor region comes from host memory).
 * flags: DS_FILE_DIRECT / DS_FILE_SYNC / DS_FILE_URING as for a flush.  The plan must outlive
 * the ds_ckpt.  Errors: DS_EINVAL, DS_ENOMEM, DS_EIO.
 */
int ds_ckpt_create(const char *path, const ds_plan *plan, uint32_t flags, ds_ckpt **out);

/* The writer of file `file` of a plan of several files (for a plan of one file,
 * ds_ckpt_create_part(path, plan, 0, ...) is ds_ckpt_create, which refuses a plan
 * of several).  Errors: as ds_ckpt_create. */
int ds_ckpt_create_part(const char *path, const ds_plan *plan, uint32_t file, uint32_t flags, ds_ckpt **out);

/* Fills the tensor regions of ALL files of a plan of several files from one
 * snapshot of that plan: parts[f] must be the writer of file f, n_parts the
 * plan's number of files; one flush with `threads` writers serves them all.
 * Flags are those of parts[0].  Each part is then finished on its own with
 * ds_ckpt_finish, in any order; the first of these calls waits for the flush,
 * and every part must be finished.  Errors: DS_EINVAL, DS_ESTATE, DS_ENOMEM. */
int ds_ckpt_flush_snapshot_parts(ds_ckpt *const *parts, uint32_t n_parts, ds_event *snapshot, uint32_t threads);

/* Fills the tensor region from a snapshot of the same plan: ds_flush_start on
 * this file (`threads` writers).  Once per ds_ckpt; returns at once.
 * Errors: DS_EINVAL, DS_ESTATE (a second call), DS_ENOMEM. */
int ds_ckpt_flush_snapshot(ds_ckpt *ckpt, ds_event *snapshot, uint32_t threads);

/* Writes len bytes of HOST memory at file_off of the tensor region
 * (file_off + len <= T).  Thread-safe.  Errors: DS_EINVAL, DS_ERANGE, DS_EIO. */
int ds_ckpt_write_region(ds_ckpt *ckpt, uint64_t file_off, const void *host, uint64_t len);

/*
 * Appends one chunk of a serialized object to the log.  Thread-safe and
 * concurrent with the flush of the tensors: the position is claimed with one
 * atomic add, then written.  Chunks of one object_id are numbered in call
 * order.  len may be 0 (data may then be NULL).  Errors: DS_EINVAL, DS_EIO.
 */
int ds_ckpt_append(ds_ckpt *ckpt, uint64_t object_id, const void *data, uint64_t len);

/*
 * An object state provider (Sec. V-A3): an iterator that presents the next chunk
 * of an object's serialized stream -- how many bytes, from where.  Returns 1 with
 * *data / *len set (the bytes stay valid until the next call), 0 at the end of
 * the stream, or a negative value to stop with that value as the error.
 */
typedef int (*ds_chunk_provider)(void *ctx, const void **data, uint64_t *len);

/* Drains `next` into the log: one ds_ckpt_append per chunk, in the order
 * presented, so the serializer never has to hold the whole object.  Several
 * threads may drain providers of different objects into one ds_ckpt at once.
 * *n_chunks (may be NULL) = chunks appended.  Errors: DS_EINVAL, DS_EIO, or the
 * provider's own negative value. */
int ds_ckpt_append_from(ds_ckpt *ckpt, uint64_t object_id, ds_chunk_provider next, void *ctx, uint64_t *n_chunks);

/*
 * Waits for the flush (if one was started), writes trailer and footer, syncs
 * under DS_FILE_SYNC, closes the file and frees the ds_ckpt (also on error).
 * No ds_ckpt_append may be running.  Out pointers may be NULL: the file's
 * length, seconds since ds_ckpt_create.  Errors: DS_EIO, or the error that
 * ended the snapshot / the first failed append.
 */
int ds_ckpt_finish(ds_ckpt *ckpt, uint64_t *file_bytes, double *seconds);

typedef struct ds_ckpt_layout {
  uint64_t align;
  uint64_t tensor_bytes;   /* T                              */
  uint64_t log_end;        /* E: where the trailer starts    */
  uint64_t n_tensors;
  uint64_t n_chunks;       /* log chunks                     */
  uint64_t n_objects;      /* distinct object ids            */
  uint64_t file_bytes;
} ds_ckpt_layout;

typedef struct ds_ckpt_tensor {
  uint64_t tensor_id;
  uint32_t dtype;
  uint32_t ndim;
  int64_t shape[DS_MAX_DIMS];
  uint64_t file_offset;
  uint64_t nbytes;
} ds_ckpt_tensor;

/*
 * Opens a checkpoint file and checks it: footer magic, version and checksum,
 * trailer bounds and checksum, every tensor inside [0, T) at a multiple of the
 * alignment, every chunk inside [T, E), chunk order and numbering.
 * Errors: DS_EIO (cannot open / read), DS_EFORMAT, DS_ENOMEM.
 */
int ds_ckpt_open(const char *path, ds_ckpt_reader **out);
int ds_ckpt_close(ds_ckpt_reader *reader);
int ds_ckpt_layout_info(const ds_ckpt_reader *reader, ds_ckpt_layout *out);
/* Tensor entry i (0 <= i < n_tensors). */
int ds_ckpt_tensor_info(const ds_ckpt_reader *reader, size_t i, ds_ckpt_tensor *out);
/* The k-th object in ascending id order (0 <= k < n_objects): its id and length. */
int ds_ckpt_object_at(const ds_ckpt_reader *reader, size_t k, uint64_t *object_id, uint64_t *nbytes);
/* Reads object `object_id` whole into buf (capacity cap); *len = its length.
 * Errors: DS_EINVAL (no such object), DS_ERANGE (cap too small; *len is set), DS_EIO. */
int ds_ckpt_object_read(const ds_ckpt_reader *reader, uint64_t object_id, void *buf, uint64_t cap, uint64_t *len);
/* DS_OK if the file's tensor entries, alignment and T are exactly the plan's
 * manifest (ids, dtypes, shapes, offsets, sizes, order); DS_EFORMAT if not. */
int ds_ckpt_matches_plan(const ds_ckpt_reader *reader, const ds_plan *plan);
/* ds_ckpt_matches_plan, then ds_restore_from_file on the tensor region. */
int ds_ckpt_restore(const ds_ckpt_reader *reader, ds_engine *engine, const ds_plan *plan, uint32_t threads,
                    uint32_t flags, void *compute_stream, ds_event **out);
/* The same for file `file` of a plan of several files: T is that file's region,
 * the entries are the plan's entries of that file.  ds_ckpt_matches_plan is part 0
 * of a plan of one file (DS_EINVAL for a plan of several). */
int ds_ckpt_matches_plan_part(const ds_ckpt_reader *reader, const ds_plan *plan, uint32_t file);
/* Every reader checked against its part (readers[f] = file f, n_parts = the
 * plan's number of files), then ONE restore of the whole rank out of all files
 * (ds_restore_from_files on the tensor regions).  Errors: DS_EINVAL, DS_EFORMAT,
 * and those of ds_restore_from_file. */
int ds_ckpt_restore_parts(const ds_ckpt_reader *const *readers, uint32_t n_parts, ds_engine *engine,
                          const ds_plan *plan, uint32_t threads, uint32_t flags, void *compute_stream,
                          ds_event **out);

/* ---- misc ---------------------------------------------------------------- */

const char *ds_strerror(int code);

/* hipError_t of the HIP call that last produced DS_EHIP on this thread. */
int ds_last_hip_error(void);

/*
 * Measurement aid, not part of the method: a plain contiguous device-to-device
 * copy of nbytes (multiple of 16; both pointers 16-byte aligned, device
 * memory, not overlapping) with the same launch shape and memory instructions
 * as the gather kernel.  It gives the HBM rate a pure copy reaches on this
 * GPU, against which the gather is reported, and a kernel of known traffic to
 * scale hardware byte counters with.  Asynchronous on `stream`.
 * Errors: DS_EINVAL, DS_ERANGE, DS_EHIP.
 */
int ds_copy_probe(void *dst_dev, const void *src_dev, uint64_t nbytes, void *stream);

/*
 * For differential snapshots (the data reduction the paper's conclusions name as
 * future work; an experiment here, the engine does not use it): compares two
 * images of nbytes (multiple of 16; both pointers device memory, 16-byte
 * aligned) block by block and sets changed_dev[k] (device memory, one uint32 per
 * block, ceil(nbytes / block_bytes) of them) to 1 if block k differs anywhere,
 * else to 0.  block_bytes: a power of two >= 16 KiB.  Asynchronous on `stream`.
 * Errors: DS_EINVAL, DS_ERANGE, DS_EHIP.
 */
int ds_image_diff(const void *image_a_dev, const void *image_b_dev, uint64_t nbytes, uint64_t block_bytes,
                  uint32_t *changed_dev, void *stream);

/*
 * For compressed snapshots (the other data reduction the paper's conclusions name
 * as future work; an experiment here, the engine does not use it): block elision.
 * The image (nbytes, a multiple of 16; device memory, 16-byte aligned) is cut into
 * blocks of block_bytes (a power of two >= 16 KiB; the last block may be short).
 * A block all of whose 16-byte units equal its first one (zero padding,
 * zero-initialised optimizer moments, fills whose period divides 16) is CONSTANT
 * and is replaced by that unit.  Outputs, all device memory of the caller:
 *   keep_dev[k]      1 if block k is stored whole, 0 if it is constant (n_blocks x u32)
 *   pos_dev[k]       kept blocks before block k; pos_dev[n_blocks] = their number
 *                    (n_blocks + 1 x u32)
 *   patterns_dev     the first 16 bytes of every block (n_blocks x 16 bytes)
 *   packed_dev       the kept blocks one behind the other, block k in the slot of
 *                    block_bytes at pos_dev[k] * block_bytes (capacity: n_blocks slots;
 *                    of a short last block only its own bytes are written)
 * What has to leave the device is pos_dev[n_blocks] slots of packed_dev, the
 * patterns and the flags.  Asynchronous on `stream`.  The paper gives no scheme:
 * this one is the library's, defined by oracle/image_compress.py for the tests.
 * Errors: DS_EINVAL, DS_ERANGE, DS_EHIP.
 */
int ds_image_compress(const void *image_dev, uint64_t nbytes, uint64_t block_bytes, uint32_t *keep_dev,
                      uint32_t *pos_dev, void *patterns_dev, void *packed_dev, void *stream);

/*
 * Tunables for experiments, read when a plan is created / a kernel launched:
 *   "chunk_bytes"   image bytes per work-group chunk: 8, 16 (default) or 32 KiB
 *   "variant"       0 = default (non-temporal accesses; the lean gather writes the image with
 *                   write-through streaming buffer stores), 1 = plain loads and stores,
 *                   2 = non-temporal global loads and stores everywhere, 3 = default accesses but
 *                   work-group i takes chunk i (no XCD-contiguous order), 4 = default, but plans made
 *                   under it do not mark chunks for the gather's aligned-load route (tensors at
 *                   addresses that are not multiples of 16 are then read with unaligned loads),
 *                   5 = default, but a plan in which most chunks take the general path is launched
 *                   with four wavefronts per SIMD like any other (by default it gets five for the
 *                   gather and six for the scatter)
 *   "grid_limit"    work-groups per launch of ds_pack / ds_unpack (each then walks several chunks);
 *                   0 = one per chunk (default).  Engines have their own pack_grid_limit
 *   "drop_pinned_cache"   (set only) a non-zero value frees the pinned ring and the device staging the
 *                   library keeps from the last destroyed engine for the next one (see ds_engine_create)
 *   "io_uring_available"  (get only) 1 if this process can set up an io_uring, else 0
 * Returns DS_EINVAL for an unknown key or a value out of range.
 */
int ds_config_set(const char *key, uint64_t value);
int ds_config_get(const char *key, uint64_t *value);

#ifdef __cplusplus
}
#endif
#endif /* DATASTATES_H */
