// Device-side structures and helpers shared by the xorenc kernels (arXiv 1905.10138).
#ifndef XORENC_DEVICE_H
#define XORENC_DEVICE_H

#include <hip/hip_runtime.h>

#include "xorenc_internal.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

struct DevLayer {
  const uint8_t *enc;
  const uint32_t *mask32;  // the uint64 mask words seen as pairs of 32-bit halves
  const uint32_t *patch_off;
  const uint16_t *patch;
  const float *alpha;
  int32_t m, n, spr, nrb, n_units, nib, q;  // nib = ceil(n_in/8): byte-indexed XOR tables per word
  int32_t n_in;
  int32_t J, espr;  // 64-bit words per slice (n_out/64), slices per row
  int64_t n_slots, n_eslots;
  // Launches that split the reduction dimension over several workgroups per output tile: partial tiles
  // (kSplitTileFloats floats per workgroup, at most kSplitMaxGroups workgroups) and one arrival counter per
  // output tile, zero between launches.  Filled by xorenc_spmm from the library's own scratch area.
  float *split_part;
  uint32_t *split_ticket;
  // column j of M restricted to word w of a slice (rows 64 w .. 64 w + 63): lower and upper 32 rows
  uint32_t Mcol_lo[XORENC_MAX_J * XORENC_MAX_N_IN];
  uint32_t Mcol_hi[XORENC_MAX_J * XORENC_MAX_N_IN];
};


constexpr int kSplitTileFloats = 4096;  // largest output tile of a split launch (64 x 64)
constexpr int kSplitMaxGroups = 256;    // workgroups of a split launch (one per CU)

// field `e` (n_in bits at bit e*n_in) of the encrypted bit stream, seen as aligned dwords
static __device__ inline uint32_t load_enc(const uint8_t *enc, int64_t e, int n_in) {
  const uint32_t *d = reinterpret_cast<const uint32_t *>(enc);
  const int64_t bit = e * n_in;
  const int64_t i = bit >> 5;
  const int sh = (int)(bit & 31);
  uint32_t x = d[i] >> sh;
  if (sh + n_in > 32) x |= d[i + 1] << (32 - sh);
  return n_in < 32 ? (x & ((1u << n_in) - 1u)) : x;
}

// Lanes 32k .. 32k+31 hold the fields of the 32 slices of one unit (x, n_in bits each, field index
// e0 + lane%32 with e0 a multiple of 32): write the unit's n_in dwords of the stream.  Every lane
// of the wave must call this; lanes whose `valid` is false write nothing.
static __device__ inline void store_enc_unit(uint8_t *enc, int64_t e, int n_in, uint32_t x, bool valid) {
  const int rr = (int)(threadIdx.x & 31);
  const int lo_bit = 32 * rr;             // this lane composes dword rr of the run (if rr < n_in)
  const int first = lo_bit / n_in;        // first field that reaches into it
  uint32_t word = 0;
  const int span = 32 / n_in + 2;         // fields that can overlap one dword
  for (int t = 0; t < span; ++t) {        // uniform
    const int k = first + t;
    const uint32_t xk = (uint32_t)__shfl((int)x, k & 31, 32);
    const int pos = k * n_in - lo_bit;    // where field k starts relative to this dword
    if (k < 32 && pos < 32) word |= pos >= 0 ? (xk << pos) : (xk >> (-pos));
  }
  if (valid && rr < n_in) {
    uint32_t *d = reinterpret_cast<uint32_t *>(enc);
    d[((e - rr) >> 5) * n_in + rr] = word;
  }
}

static __device__ inline uint32_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// Validates a caller's layer descriptor (host) and fills the kernel-argument form of it.
int32_t xorenc_fill_dev_layer(const xorenc_layer *layer, DevLayer *D);

#endif
