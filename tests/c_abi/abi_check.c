/* A plain C user of the library: includes the public header, prints the sizes
 * and field offsets of its structs (the test compares them with the Python
 * binding's mirrors), then runs the host-only part of the interface -- layout,
 * a host-only plan, a checkpoint file written from host memory and read back.
 * No device call is made. */
#include <stddef.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "datastates.h"

#define CHECK(x)                                                         \
  do {                                                                   \
    int rc_ = (x);                                                       \
    if (rc_ != DS_OK) {                                                  \
      fprintf(stderr, "%s -> %d (%s)\n", #x, rc_, ds_strerror(rc_));     \
      return 1;                                                          \
    }                                                                    \
  } while (0)

int main(int argc, char **argv) {
  const char *path = argc > 1 ? argv[1] : "/tmp/abi_check.ckpt";
  printf("sizeof ds_shard_desc %zu\n", sizeof(ds_shard_desc));
  printf("offsetof ds_shard_desc.shape %zu\n", offsetof(ds_shard_desc, shape));
  printf("offsetof ds_shard_desc.strides %zu\n", offsetof(ds_shard_desc, strides));
  printf("offsetof ds_shard_desc.tensor_id %zu\n", offsetof(ds_shard_desc, tensor_id));
  printf("offsetof ds_shard_desc.file_offset %zu\n", offsetof(ds_shard_desc, file_offset));
  printf("sizeof ds_plan_stats %zu\n", sizeof(ds_plan_stats));
  printf("sizeof ds_engine_opts %zu\n", sizeof(ds_engine_opts));
  printf("offsetof ds_engine_opts.first_launch_bytes %zu\n", offsetof(ds_engine_opts, first_launch_bytes));
  printf("sizeof ds_snapshot_stats %zu\n", sizeof(ds_snapshot_stats));
  printf("sizeof ds_ckpt_layout %zu\n", sizeof(ds_ckpt_layout));
  printf("sizeof ds_ckpt_tensor %zu\n", sizeof(ds_ckpt_tensor));
  printf("offsetof ds_ckpt_tensor.file_offset %zu\n", offsetof(ds_ckpt_tensor, file_offset));

  /* three shards over a host buffer: a contiguous vector, a 2-D view with a pitch, a scalar */
  static float parent[64 * 48];
  for (int i = 0; i < 64 * 48; ++i) parent[i] = (float)i;
  ds_shard_desc d[3];
  memset(d, 0, sizeof d);
  d[0].base = parent;      d[0].dtype = DS_F32; d[0].ndim = 1; d[0].shape[0] = 100; d[0].strides[0] = 1; d[0].tensor_id = 11;
  d[1].base = parent + 7;  d[1].dtype = DS_F32; d[1].ndim = 2; d[1].shape[0] = 30; d[1].shape[1] = 20;
  d[1].strides[0] = 48;    d[1].strides[1] = 1;  d[1].tensor_id = 12;
  d[2].base = parent + 5;  d[2].dtype = DS_F32; d[2].ndim = 0; d[2].tensor_id = 13;
  uint64_t total = 0;
  CHECK(ds_layout_assign(d, 3, 256, &total));
  printf("total %llu offsets %llu %llu %llu\n", (unsigned long long)total, (unsigned long long)d[0].file_offset,
         (unsigned long long)d[1].file_offset, (unsigned long long)d[2].file_offset);
  ds_plan *plan = NULL;
  CHECK(ds_plan_create(d, 3, 256, DS_PLAN_HOST_ONLY | DS_PLAN_STRICT, &plan));
  ds_plan_stats st;
  CHECK(ds_plan_info(plan, &st));
  printf("payload %llu shards %llu strided %llu\n", (unsigned long long)st.payload_bytes,
         (unsigned long long)st.n_shards, (unsigned long long)st.n_strided);

  /* the image, written by hand from the definition: row-major order of each view, zero padding */
  unsigned char *image = calloc(total, 1);
  memcpy(image + d[0].file_offset, parent, 400);
  for (int r = 0; r < 30; ++r) memcpy(image + d[1].file_offset + 80 * r, parent + 7 + 48 * r, 80);
  memcpy(image + d[2].file_offset, parent + 5, 4);

  ds_ckpt *ck = NULL;
  CHECK(ds_ckpt_create(path, plan, 0, &ck));
  CHECK(ds_ckpt_write_region(ck, 0, image, total));
  CHECK(ds_ckpt_append(ck, 42, "hello ", 6));
  CHECK(ds_ckpt_append(ck, 7, "x", 1));
  CHECK(ds_ckpt_append(ck, 42, "world", 5));
  uint64_t file_bytes = 0;
  CHECK(ds_ckpt_finish(ck, &file_bytes, NULL));

  ds_ckpt_reader *rd = NULL;
  CHECK(ds_ckpt_open(path, &rd));
  ds_ckpt_layout lay;
  CHECK(ds_ckpt_layout_info(rd, &lay));
  CHECK(ds_ckpt_matches_plan(rd, plan));
  char buf[32] = {0};
  uint64_t len = 0;
  CHECK(ds_ckpt_object_read(rd, 42, buf, sizeof buf, &len));
  ds_ckpt_tensor t;
  CHECK(ds_ckpt_tensor_info(rd, 1, &t));
  printf("file %llu tensors %llu objects %llu chunks %llu object42 '%.*s' tensor1 id %llu ndim %u shape %lld %lld\n",
         (unsigned long long)file_bytes, (unsigned long long)lay.n_tensors, (unsigned long long)lay.n_objects,
         (unsigned long long)lay.n_chunks, (int)len, buf, (unsigned long long)t.tensor_id, t.ndim,
         (long long)t.shape[0], (long long)t.shape[1]);
  CHECK(ds_ckpt_close(rd));
  CHECK(ds_plan_destroy(plan));
  free(image);
  return 0;
}
