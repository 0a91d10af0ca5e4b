// Sixteen bytes taken at any byte position out of two 16-byte units: what the kernels use to
// assemble (gather) or split (scatter) an image unit that is cut by the end of a contiguous run.
//
// Written on 32-bit words only: the position picks words with selects, the sub-word part is one
// byte-alignment per output word.  No shift of a 64-bit value by a run-time count anywhere (an
// earlier form built the result from four such shifts).
//
// The file compiles for the device and, unchanged, for the host: a CPU test includes it and checks
// every position against a byte loop.  Only ds_align_bytes differs between the two: the device
// takes the byte-align instruction, the host the same definition written with shifts.
#pragma once

#include <stdint.h>

#if defined(__HIPCC__)
#define DS_SPLICE_FN __host__ __device__ __forceinline__
#else
#define DS_SPLICE_FN static inline
#endif

// Bytes [r, r+4) of the eight bytes lo || hi (lo holds bytes 0..3, little-endian), r = 0..3.
DS_SPLICE_FN uint32_t ds_align_bytes(uint32_t hi, uint32_t lo, uint32_t r) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __builtin_amdgcn_alignbyte(hi, lo, r);
#else
  return r ? (lo >> (8u * r)) | (hi << (32u - 8u * r)) : lo;
#endif
}

struct DsWords4 {
  uint32_t w[4];
};

// Bytes [s, s+16) of the 32 bytes a || b, 0 <= s < 16.
DS_SPLICE_FN DsWords4 ds_splice_words(DsWords4 a, DsWords4 b, uint32_t s) {
  uint32_t w0 = a.w[0], w1 = a.w[1], w2 = a.w[2], w3 = a.w[3];
  uint32_t w4 = b.w[0], w5 = b.w[1], w6 = b.w[2], w7 = b.w[3];
  if (s & 8u) {  // the result starts two words further on
    w0 = w2; w1 = w3; w2 = w4; w3 = w5; w4 = w6; w5 = w7;
  }
  if (s & 4u) {  // ... and one more
    w0 = w1; w1 = w2; w2 = w3; w3 = w4; w4 = w5;
  }
  const uint32_t r = s & 3u;  // now it starts in byte r of w0 and ends in w4
  DsWords4 out;
  out.w[0] = ds_align_bytes(w1, w0, r);
  out.w[1] = ds_align_bytes(w2, w1, r);
  out.w[2] = ds_align_bytes(w3, w2, r);
  out.w[3] = ds_align_bytes(w4, w3, r);
  return out;
}
