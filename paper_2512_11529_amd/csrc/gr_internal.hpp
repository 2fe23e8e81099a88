// Internal helpers shared by the HIP translation units of libgr (gfx950 only).  Not part of the ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "gr.h"

#define GR_HIP_TRY(expr)                          \
  do {                                            \
    hipError_t e_ = (expr);                       \
    if (e_ != hipSuccess) return GR_ERR_HIP;      \
  } while (0)

static inline size_t gr_align256(size_t n) { return (n + 255) & ~(size_t)255; }

// ------------------------------------------------------------------ mask blob layout
// One contiguous, position-independent blob.  All offsets are bytes from the blob start.
//   l0        uint32[words]            bit v set <=> some item starts with v
//   l1        uint32[V][words]         bit t2 of row t1 set <=> some item starts with (t1, t2)
//   off1      int32[V+1]               first table row whose first token is >= t
//   pair_off  int32[V+1]               first (t1,t2) pair whose first token is >= t
//   pair_t2   int32[n_pairs]           second token of every distinct (t1,t2) pair, table order
//   pair_row  int32[n_pairs+1]         first table row of every pair; pair_row[n_pairs] = n_items
//   t3        int32[n_items]           third column of the table
#define GR_MASK_MAGIC 0x4d524758u /* "XGRM" */
struct gr_mask_header {
  uint32_t magic;
  int32_t V, depth, words;     // words = ceil(V / 32)
  int64_t n_items;
  int64_t n_pairs;             // written on the device by the build
  int64_t off_l0, off_l1, off_off1, off_pair_off, off_pair_t2, off_pair_row, off_t3, total_bytes;
};

static inline void gr_mask_layout(int64_t n_items, int32_t V, gr_mask_header* h) {
  h->magic = GR_MASK_MAGIC;
  h->V = V;
  h->depth = 3;
  h->words = (V + 31) / 32;
  h->n_items = n_items;
  h->n_pairs = 0;
  size_t o = 256;
  h->off_l0 = (int64_t)o;       o += gr_align256((size_t)h->words * 4);
  h->off_l1 = (int64_t)o;       o += gr_align256((size_t)V * h->words * 4);
  h->off_off1 = (int64_t)o;     o += gr_align256((size_t)(V + 1) * 4);
  h->off_pair_off = (int64_t)o; o += gr_align256((size_t)(V + 1) * 4);
  h->off_pair_t2 = (int64_t)o;  o += gr_align256((size_t)n_items * 4);
  h->off_pair_row = (int64_t)o; o += gr_align256((size_t)(n_items + 1) * 4);
  h->off_t3 = (int64_t)o;       o += gr_align256((size_t)n_items * 4);
  h->total_bytes = (int64_t)o;
}

#ifdef __HIPCC__
// ------------------------------------------------------------------ wave64 primitives
__device__ __forceinline__ int gr_lane() { return (int)__lane_id(); }

__device__ __forceinline__ float gr_wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ double gr_wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ uint32_t gr_wave_sum_u32(uint32_t v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Order-preserving map fp32 -> uint32 (larger float <=> larger key); no NaN expected.
__device__ __forceinline__ uint32_t gr_ordkey(float f) {
  uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float gr_ordkey_inv(uint32_t k) {
  uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
  return __uint_as_float(u);
}
#endif
