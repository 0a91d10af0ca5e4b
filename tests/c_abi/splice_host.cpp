// Host build of the kernels' splice routine (csrc/ds_splice.h, included unchanged), for the CPU test
// that checks every position against a byte loop.
#include <string.h>

#include "ds_splice.h"

extern "C" void splice_host(const unsigned char a[16], const unsigned char b[16], unsigned s, unsigned char out[16]) {
  DsWords4 wa, wb;
  memcpy(wa.w, a, 16);
  memcpy(wb.w, b, 16);
  const DsWords4 r = ds_splice_words(wa, wb, s);
  memcpy(out, r.w, 16);
}

extern "C" unsigned align_bytes_host(unsigned hi, unsigned lo, unsigned r) { return ds_align_bytes(hi, lo, r); }
