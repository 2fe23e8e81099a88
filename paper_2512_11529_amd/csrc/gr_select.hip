// gr_beam_select: beam item step (paper Sections 6.1-6.3) on gfx950.
//
// Two kernels per call (no host synchronisation, no allocation; everything lives in caller buffers):
//   k_rows         both kinds of beam row in one launch:
//                  streamed rows, one workgroup each: validity bits staged in LDS (dense level-0 /
//                  level-1 mask rows, or the row's sparse last-level positions set in an empty mask),
//                  logits read ONCE with 16-byte loads and kept in registers for the max, the fp64
//                  sum-exp and the per-chunk maxima; the validity bits come straight from the mask row in
//                  memory, and a thinly populated row packs its valid logits before exponentiating them;
//                  gathered rows (few valid children), one wavefront each: only those logits are read.
//   k_select       one workgroup per request: top-W of the request's candidates by (score descending,
//                  flat index ascending).  It never sorts the W*V candidates: the rows kernels leave
//                  one "chunk key" (best candidate score) per 1/256th of a row; a histogram of those
//                  keys yields a threshold that at least W candidates reach, only the chunks that
//                  reach it are re-read, and only their candidates above the threshold are sorted
//                  (the early-termination idea of Section 6.2: stop as soon as the survivors are
//                  fixed).  If the survivors do not fit in LDS (massive ties) an exact MSB radix
//                  select over all candidates takes over.
//
// Arithmetic that decides beam order is fixed: m = fp32 max over valid logits, S = fp64 sum of
// exp(x - m), lse = fp32(m + log S), bias = score_in - lse (fp32), cand = bias + x (fp32), with no
// fused multiply-add in the last two operations.
#include "gr_internal.hpp"

namespace {

constexpr int kRowThreads = 256;
constexpr int kChunksPerRow = 256;  // chunk keys stored per row (dense rows use all, sparse rows the first 64)
constexpr int kSelThreads = 1024;
constexpr int kSparseMax = 256;     // rows with at most this many valid children are gathered, not streamed
constexpr int kSparseKeys = 64;     // chunk keys of a gathered row (chunk k = children k, k+64, ...)
constexpr int kListCap = 8192;      // survivors that fit in LDS
constexpr int kChunkCap = 2048;     // chunks re-read by the fast path
constexpr int kHistBins = 2048;
constexpr int kMaxMaskWords = 1024; // V <= 32768
constexpr int kRegV4 = 8;           // float4 per thread kept in registers (V <= 8192)
constexpr int kMaxW = 2048;
constexpr size_t kSelLdsBytes = (size_t)kListCap * 8 + (size_t)kHistBins * 4 + (size_t)kChunkCap * 4 + (size_t)kMaxW * 20;

enum { ROW_DEAD = 0, ROW_DENSE = 1, ROW_SPARSE = 2 };

struct SelCtx {
  int B, W, V, depth, step, flags;
  int vec4;                  // V % 4 == 0: rows are 16-byte aligned, chunks interleave float4 groups
  int epc;                   // element slots per chunk of a dense row
  const char* blob;          // mask blob or nullptr
  const float* logits;
  const float* scores_in;
  const int32_t* prefix_in;
  const int32_t* range_in;
  int32_t* parent_out;
  int32_t* token_out;
  float* scores_out;
  int32_t* prefix_out;
  int32_t* range_out;
  int32_t* item_index_out;
  float* row_bias;           // workspace [B*W]
  int32_t* row_mode;         // workspace [B*W]
  float* row_top;            // workspace [B*W]: best candidate score of the row (= its largest chunk key)
  float* chunk_key;          // workspace [B*W*kChunksPerRow]
};

struct MaskView {
  const uint32_t* l0;
  const uint32_t* l1;
  const int32_t* off1;
  const int32_t* pair_off;
  const int32_t* pair_t2;
  const int32_t* pair_row;
  const int32_t* t3;
  int words;
  int64_t n_items;
  bool ok;                   // header matches the call (magic, V, depth)
};

__device__ __forceinline__ MaskView mask_view(const char* blob, int V, int depth) {
  const gr_mask_header* h = (const gr_mask_header*)blob;
  MaskView m;
  m.l0 = (const uint32_t*)(blob + h->off_l0);
  m.l1 = (const uint32_t*)(blob + h->off_l1);
  m.off1 = (const int32_t*)(blob + h->off_off1);
  m.pair_off = (const int32_t*)(blob + h->off_pair_off);
  m.pair_t2 = (const int32_t*)(blob + h->off_pair_t2);
  m.pair_row = (const int32_t*)(blob + h->off_pair_row);
  m.t3 = (const int32_t*)(blob + h->off_t3);
  m.words = h->words;
  m.n_items = h->n_items;
  m.ok = h->magic == GR_MASK_MAGIC && h->V == V && h->depth == depth;
  return m;
}

// The valid children of a beam row as a sorted token list (steps 1 and 2).  A prefix or range that
// this mask could not have produced yields an empty list instead of an out-of-bounds read.
__device__ __forceinline__ void row_children(const SelCtx& c, const MaskView& mv, int row, const int32_t** list, int* n) {
  if (!mv.ok) { *list = nullptr; *n = 0; return; }
  if (c.step == 1) {
    const int t1 = c.prefix_in[(size_t)row * c.depth];
    const bool ok = t1 >= 0 && t1 < c.V;
    const int p0 = ok ? mv.pair_off[t1] : 0, p1 = ok ? mv.pair_off[t1 + 1] : 0;
    *list = mv.pair_t2 + p0;
    *n = p1 - p0;
  } else {
    int lo = c.range_in[2 * (size_t)row], hi = c.range_in[2 * (size_t)row + 1];
    if (lo < 0 || hi < lo || (int64_t)hi > mv.n_items) { lo = 0; hi = 0; }
    *list = mv.t3 + lo;
    *n = hi - lo;
  }
}

// Does this row get gathered (true) or streamed (false)?  Same decision in every kernel.
__device__ __forceinline__ bool row_is_sparse(const SelCtx& c, int n_children) {
  return c.blob && c.step >= 1 && !(c.flags & GR_SELECT_FORCE_DENSE) && n_children <= kSparseMax;
}

// Token held by element slot e of chunk k of a dense row (or >= V when the slot is empty).
__device__ __forceinline__ int dense_slot_token(const SelCtx& c, int k, int e) {
  return c.vec4 ? 4 * (k + kChunksPerRow * (e >> 2)) + (e & 3) : k + kChunksPerRow * e;
}

__device__ __forceinline__ int lower_bound_i32(const int32_t* a, int n, int key) {
  int lo = 0, hi = n;
  while (lo < hi) { int mid = (lo + hi) >> 1; if (a[mid] < key) lo = mid + 1; else hi = mid; }
  return lo;
}

// e^(x - ref) in fp64 for fp32 x <= ref (and not more than ~700 below it), about 1e-14 relative:
//   t = (x - ref) * 64/ln2 = n + f with n = rint(t), |f| <= 1/2, both from one addition of 1.5 * 2^52 (the sum's
//   low word then holds n); e^(x-ref) = 2^(n>>6) * 2^((n&63)/64) * 2^(f/64) with
//   2^(f/64) - 1 = f (c1 + f (c2 + f (c3 + f c4))), c_k = (ln2/64)^k / k!  (truncation < 4e-14), the middle factor
//   from a 64-entry table in LDS and the power of two added to the exponent field.  Eleven fp64 and four integer
//   operations, all at the full rate (no rounding, conversion-to-integer or ldexp instruction).  The error is far
//   below what the single fp32 rounding of lse = m + log S can see.
// The constants live in scalar registers (set up once per kernel): left to itself the compiler
// re-materialises each 64-bit literal with vector moves next to every use.
struct ExpK { double c, magic, c1, c2, c3, c4; };
__device__ __forceinline__ ExpK exp_consts() {
  ExpK k = {0x1.71547652b82fep+6, 0x1.8p+52, 0x1.62e42fefa39efp-7, 0x1.ebfbdff82c58fp-15, 0x1.c6b08d704a0c0p-23,
            0x1.3b2ab6fba4e77p-31};
  asm volatile("" : "+s"(k.c), "+s"(k.magic), "+s"(k.c1), "+s"(k.c2), "+s"(k.c3), "+s"(k.c4));
  return k;
}
__constant__ double c_exp_tab[64] = {        // 2^(j/64), correctly rounded
    0x1.0000000000000p+0, 0x1.02c9a3e778061p+0, 0x1.059b0d3158574p+0, 0x1.0874518759bc8p+0,
    0x1.0b5586cf9890fp+0, 0x1.0e3ec32d3d1a2p+0, 0x1.11301d0125b51p+0, 0x1.1429aaea92de0p+0,
    0x1.172b83c7d517bp+0, 0x1.1a35beb6fcb75p+0, 0x1.1d4873168b9aap+0, 0x1.2063b88628cd6p+0,
    0x1.2387a6e756238p+0, 0x1.26b4565e27cddp+0, 0x1.29e9df51fdee1p+0, 0x1.2d285a6e4030bp+0,
    0x1.306fe0a31b715p+0, 0x1.33c08b26416ffp+0, 0x1.371a7373aa9cbp+0, 0x1.3a7db34e59ff7p+0,
    0x1.3dea64c123422p+0, 0x1.4160a21f72e2ap+0, 0x1.44e086061892dp+0, 0x1.486a2b5c13cd0p+0,
    0x1.4bfdad5362a27p+0, 0x1.4f9b2769d2ca7p+0, 0x1.5342b569d4f82p+0, 0x1.56f4736b527dap+0,
    0x1.5ab07dd485429p+0, 0x1.5e76f15ad2148p+0, 0x1.6247eb03a5585p+0, 0x1.6623882552225p+0,
    0x1.6a09e667f3bcdp+0, 0x1.6dfb23c651a2fp+0, 0x1.71f75e8ec5f74p+0, 0x1.75feb564267c9p+0,
    0x1.7a11473eb0187p+0, 0x1.7e2f336cf4e62p+0, 0x1.82589994cce13p+0, 0x1.868d99b4492edp+0,
    0x1.8ace5422aa0dbp+0, 0x1.8f1ae99157736p+0, 0x1.93737b0cdc5e5p+0, 0x1.97d829fde4e50p+0,
    0x1.9c49182a3f090p+0, 0x1.a0c667b5de565p+0, 0x1.a5503b23e255dp+0, 0x1.a9e6b5579fdbfp+0,
    0x1.ae89f995ad3adp+0, 0x1.b33a2b84f15fbp+0, 0x1.b7f76f2fb5e47p+0, 0x1.bcc1e904bc1d2p+0,
    0x1.c199bdd85529cp+0, 0x1.c67f12e57d14bp+0, 0x1.cb720dcef9069p+0, 0x1.d072d4a07897cp+0,
    0x1.d5818dcfba487p+0, 0x1.da9e603db3285p+0, 0x1.dfc97337b9b5fp+0, 0x1.e502ee78b3ff6p+0,
    0x1.ea4afa2a490dap+0, 0x1.efa1bee615a27p+0, 0x1.f50765b6e4540p+0, 0x1.fa7c1819e90d8p+0};
// rc = -(double)ref * k.c; x must be >= ref - 600 (callers clamp: what is cut off is below 1e-260 of the sum)
__device__ __forceinline__ double exp_rel(float x, double rc, const double* tab, const ExpK& k) {
  const double t = fma((double)x, k.c, rc);
  const double u = t + k.magic;
  const int n = __double2loint(u);
  const double f = t - (u - k.magic);
  double p = fma(f, k.c4, k.c3);
  p = fma(p, f, k.c2);
  p = fma(p, f, k.c1);
  p = p * f;
  const double tj = tab[n & 63];
  const double r = fma(tj, p, tj);
  return __hiloint2double(__double2hiint(r) + ((n >> 6) << 20), __double2loint(r));
}
// max without the NaN-quieting instructions fmaxf() drags in (NaN inputs are outside the contract)
__device__ __forceinline__ float max_raw(float a, float b) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}

// Workgroup reductions with ONE barrier each: the per-wavefront partials go to one of two slot sets, used
// alternately (every thread makes the same sequence of calls: `par` counts them), so a wavefront that is
// already writing the next reduction's partials cannot disturb a slower one that still reads this one's; the
// set after that is only written behind the next reduction's barrier.  s_red holds 2 * NWAVES entries.
template <int NWAVES>
__device__ __forceinline__ float block_max(float v, float* s_red, int& par) {
  v = gr_wave_max(v);
  float* slot = s_red + (par++ & 1) * NWAVES;
  if (gr_lane() == 0) slot[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = slot[0];
#pragma unroll
  for (int i = 1; i < NWAVES; i++) r = fmaxf(r, slot[i]);
  return r;
}
template <int NWAVES>
__device__ __forceinline__ double block_sum(double v, double* s_red, int& par) {
  v = gr_wave_sum(v);
  double* slot = s_red + (par++ & 1) * NWAVES;
  if (gr_lane() == 0) slot[threadIdx.x >> 6] = v;
  __syncthreads();
  double r = slot[0];
#pragma unroll
  for (int i = 1; i < NWAVES; i++) r += slot[i];
  return r;
}
// The same with a barrier in front as well (for callers that rely on it to publish other LDS writes).
template <int NWAVES>
__device__ __forceinline__ float block_max2(float v, float* s_red) {
  v = gr_wave_max(v);
  __syncthreads();
  if (gr_lane() == 0) s_red[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = s_red[0];
#pragma unroll
  for (int i = 1; i < NWAVES; i++) r = fmaxf(r, s_red[i]);
  return r;
}
// exclusive prefix of v over the workgroup's threads (thread order), and the total
template <int NWAVES>
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* total, uint32_t* s_red, int& par) {
  const int lane = gr_lane(), wave = threadIdx.x >> 6;
  uint32_t incl = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t t = __shfl_up(incl, o, 64);
    if (lane >= o) incl += t;
  }
  uint32_t* slot = s_red + (par++ & 1) * NWAVES;
  if (lane == 63) slot[wave] = incl;
  __syncthreads();
  uint32_t base = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < NWAVES; i++) { const uint32_t t = slot[i]; if (i < wave) base += t; tot += t; }
  *total = tot;
  return base + incl - v;
}

// ------------------------------------------------------------------------------------------------
// Rows that are streamed in full.
// ------------------------------------------------------------------------------------------------
constexpr int kQueueMax = 2048;      // valid logits of a thinly populated streamed row that are packed before exponentiation
__device__ __forceinline__ void row_dense(const SelCtx& c, int owns_dead, int row) {
  __shared__ uint32_t s_mask[kMaxMaskWords];     // (general shapes and long last-level lists only)
  __shared__ float s_q[kQueueMax];
  __shared__ float s_redf[2 * (kRowThreads / 64)];
  __shared__ double s_redd[2 * (kRowThreads / 64)];
  __shared__ uint32_t s_redu[2 * (kRowThreads / 64)];
  __shared__ double s_tab[64];
  constexpr int NW = kRowThreads / 64;
  int par = 0;
  const int tid = threadIdx.x;
  const float s_in = c.scores_in[row];
  // (the first token of the prefix picks the level-1 mask row: asked for together with the score)
  const int t1 = (c.blob && c.step == 1) ? c.prefix_in[(size_t)row * c.depth] : -1;
  if (!(s_in > -INFINITY)) {
    if (owns_dead && tid == 0) { c.row_mode[row] = ROW_DEAD; c.row_bias[row] = -INFINITY; c.row_top[row] = -INFINITY; }
    return;                                        // the keys of a dead row are never read
  }
  const int V = c.V;
  const float* x = c.logits + (size_t)row * V;
  const bool reg = c.vec4 && V <= kRegV4 * 4 * kRowThreads;
  // ---- the row is requested as early as it is known to be streamed (one HBM read: it stays in registers): at
  // once when no child count can turn it into a gathered row, else after the look-up of its children
  const int nv4 = V >> 2;
  float4 xr[kRegV4];
  auto request_row = [&]() {
#pragma unroll
    for (int i = 0; i < kRegV4; i++) {
      const int p = tid + i * kRowThreads;
      xr[i] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
      if (p < nv4) xr[i] = *(const float4*)(x + 4 * (size_t)p);
    }
  };
  const bool surely_streamed = !c.blob || c.step == 0 || (c.flags & GR_SELECT_FORCE_DENSE);
  const int32_t* list = nullptr;
  int n_list = 0;                                  // number of valid children, where it is looked up
  MaskView mv;
  mv.ok = true;
  const int words = (V + 31) >> 5;
  // the dense mask row of this beam (levels 0 and 1), or nothing (no mask, last level, mismatched blob); a row that
  // is streamed whatever its child count asks for the mask words and the logits at once
  const uint32_t* mrow = nullptr;
  uint32_t mw[kRegV4];
#pragma unroll
  for (int i = 0; i < kRegV4; i++) mw[i] = 0u;
  if (c.blob) {
    mv = mask_view(c.blob, c.V, c.depth);
    if (mv.ok) {
      if (c.step == 0) mrow = mv.l0;
      else if (c.step == 1 && t1 >= 0 && t1 < V) mrow = mv.l1 + (size_t)t1 * mv.words;
    }
    auto request_mask = [&]() {
#pragma unroll
      for (int i = 0; i < kRegV4; i++) {
        const int wi = (tid >> 3) + 32 * i;        // float4 p = tid + i * kRowThreads has its nibble in word p >> 3
        if (wi < words) mw[i] = mrow[wi];
      }
    };
    if (reg && surely_streamed) {
      if (mrow) request_mask();
      request_row();
    }
    // a level-1 row that is streamed whatever its child count needs no look-up: its mask row says what is valid
    if (c.step >= 1 && !(c.step == 1 && (c.flags & GR_SELECT_FORCE_DENSE))) {
      row_children(c, mv, row, &list, &n_list);
      if (row_is_sparse(c, n_list)) return;      // a gathered row: rows_sparse owns it
    }
    if (reg && !surely_streamed) {
      request_row();
      if (mrow) request_mask();
    }
  } else if (reg) request_row();
  // validity bits from the mask words: bit 4 i + j <-> token 4 (tid + i * kRowThreads) + j
  uint32_t mbits = 0;
#pragma unroll
  for (int i = 0; i < kRegV4; i++) mbits |= ((mw[i] >> (4 * (tid & 7))) & 0xfu) << (4 * i);
  if (tid < 64) s_tab[tid] = c_exp_tab[tid];
  const ExpK ek = exp_consts();
  // the last level has no dense mask: a long child list is set position by position in an empty LDS mask
  // (Section 6.1's sparse form applied to an existing mask); a short one is matched against directly below
  const bool lds_mask = !reg || (c.blob && c.step == 2 && n_list > 64);
  if (lds_mask) {
    if (!c.blob) {
      for (int i = tid; i < words; i += kRowThreads) s_mask[i] = 0xffffffffu;
    } else if (c.step == 2) {
      for (int i = tid; i < words; i += kRowThreads) s_mask[i] = 0u;
      __syncthreads();
      for (int i = tid; i < n_list; i += kRowThreads) { const int v = list[i]; atomicOr(&s_mask[v >> 5], 1u << (v & 31)); }
    } else {
      for (int i = tid; i < words; i += kRowThreads) s_mask[i] = mrow ? mrow[i] : 0u;
    }
  }
  __syncthreads();                                 // (s_tab, s_mask)

  float lmax = -INFINITY;     // this thread's chunk: best valid logit
  double S = 0.0;
  float m;
  if (reg) {
    // ---- validity bits straight from the mask row: bit 4 i + j <-> token 4 (tid + i * kRowThreads) + j.
    // Invalid entries become -inf: they lose every max and add nothing to the sum.
    uint32_t vbits = 0;
    if (!c.blob) {
#pragma unroll
      for (int i = 0; i < kRegV4; i++) if (tid + i * kRowThreads < nv4) vbits |= 0xfu << (4 * i);
    } else {
      if (lds_mask) {
#pragma unroll
        for (int i = 0; i < kRegV4; i++) {
          const int p = tid + i * kRowThreads;
          if (p < nv4) vbits |= ((s_mask[p >> 3] >> (4 * (p & 7))) & 0xfu) << (4 * i);
        }
      } else if (c.step == 2) {
        for (int e = 0; e < n_list; e++) {
          const int t = list[e];
          if (((t >> 2) & (kRowThreads - 1)) == tid) vbits |= 1u << (4 * (t >> 10) + (t & 3));
        }
      } else if (mrow) {
        vbits = mbits;
      }
#pragma unroll
      for (int i = 0; i < kRegV4; i++) {
        if (!((vbits >> (4 * i)) & 1u)) xr[i].x = -INFINITY;
        if (!((vbits >> (4 * i)) & 2u)) xr[i].y = -INFINITY;
        if (!((vbits >> (4 * i)) & 4u)) xr[i].z = -INFINITY;
        if (!((vbits >> (4 * i)) & 8u)) xr[i].w = -INFINITY;
      }
    }
#pragma unroll
    for (int i = 0; i < kRegV4; i++) lmax = max_raw(max_raw(max_raw(lmax, xr[i].x), max_raw(xr[i].y, xr[i].z)), xr[i].w);
    m = block_max<NW>(lmax, s_redf, par);
    if (m > -INFINITY) {
      const double rc = -(double)m * ek.c;
      const float lo = m - 600.f;
      // thinly populated row: the valid logits are packed into a queue (thread order, so the sum is
      // reproducible) and exponentiated with full lanes.  The count of valid bits decides (it equals the child
      // count where that was looked up; a row known to be well populated skips the count).
      bool queued = c.blob && c.step >= 1 && n_list <= kQueueMax;
      uint32_t total = 0, pos = 0;
      if (queued) {
        pos = block_excl_scan<NW>((uint32_t)__popc(vbits), &total, s_redu, par);
        queued = total <= (uint32_t)kQueueMax;
      }
      if (queued) {
#pragma unroll
        for (int i = 0; i < kRegV4; i++) {
          if (((vbits >> (4 * i)) & 1u) && pos < (uint32_t)kQueueMax) s_q[pos++] = xr[i].x;
          if (((vbits >> (4 * i)) & 2u) && pos < (uint32_t)kQueueMax) s_q[pos++] = xr[i].y;
          if (((vbits >> (4 * i)) & 4u) && pos < (uint32_t)kQueueMax) s_q[pos++] = xr[i].z;
          if (((vbits >> (4 * i)) & 8u) && pos < (uint32_t)kQueueMax) s_q[pos++] = xr[i].w;
        }
        __syncthreads();
        const int nq = min((int)total, kQueueMax);
        for (int i = tid; i < nq; i += kRowThreads) S += exp_rel(max_raw(s_q[i], lo), rc, s_tab, ek);
      } else {
#pragma unroll
        for (int i = 0; i < kRegV4; i++) {
          S += exp_rel(max_raw(xr[i].x, lo), rc, s_tab, ek);
          S += exp_rel(max_raw(xr[i].y, lo), rc, s_tab, ek);
          S += exp_rel(max_raw(xr[i].z, lo), rc, s_tab, ek);
          S += exp_rel(max_raw(xr[i].w, lo), rc, s_tab, ek);
          // keep the four exponentials of a load together: hoisting the first halves of all 32 costs a hundred registers
          asm volatile("" : "+v"(S)::"memory");
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
  } else {
    // general shape: two passes over the row (the second one hits in cache); same chunk layout
    const int epc = c.epc;
    for (int e = 0; e < epc; e++) {
      const int v = dense_slot_token(c, tid, e);
      if (v < V && ((s_mask[v >> 5] >> (v & 31)) & 1u)) lmax = fmaxf(lmax, x[v]);
    }
    m = block_max<NW>(lmax, s_redf, par);
    if (m > -INFINITY) {
      const double rc = -(double)m * ek.c;
      const float lo = m - 600.f;
      for (int e = 0; e < epc; e++) {
        const int v = dense_slot_token(c, tid, e);
        if (v < V && ((s_mask[v >> 5] >> (v & 31)) & 1u)) S += exp_rel(fmaxf(x[v], lo), rc, s_tab, ek);
      }
    }
  }
  if (!(m > -INFINITY)) {
    if (tid == 0) { c.row_mode[row] = ROW_DEAD; c.row_bias[row] = -INFINITY; c.row_top[row] = -INFINITY; }
    return;
  }
  S = block_sum<NW>(S, s_redd, par);
  const float lse = (float)((double)m + log(S));
  const float bias = __fsub_rn(s_in, lse);
  if (tid == 0) {
    c.row_bias[row] = bias;
    c.row_mode[row] = ROW_DENSE;
    c.row_top[row] = __fadd_rn(bias, m);
  }
  c.chunk_key[(size_t)row * kChunksPerRow + tid] = (lmax > -INFINITY) ? __fadd_rn(bias, lmax) : -INFINITY;
}

// ------------------------------------------------------------------------------------------------
// Rows with few valid children: one wavefront each, gather only the valid logits (Section 6.1's
// sparse form).  Chunk k of such a row = children k, k+64, k+128, ...
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ void rows_sparse(const SelCtx& c, int group) {
  __shared__ double s_tab[64];
  if (threadIdx.x < 64) s_tab[threadIdx.x] = c_exp_tab[threadIdx.x];
  const ExpK ek = exp_consts();
  __syncthreads();
  const int row = group * (kRowThreads / 64) + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= c.B * c.W) return;
  float* keys = c.chunk_key + (size_t)row * kChunksPerRow;
  const float s_in = c.scores_in[row];
  const MaskView mv = mask_view(c.blob, c.V, c.depth);
  const int32_t* list = nullptr;
  int n = 0;
  const bool live = s_in > -INFINITY;
  if (live) {
    row_children(c, mv, row, &list, &n);
    if (!row_is_sparse(c, n)) return;          // a streamed row: row_dense owns it
  }
  if (!live || n == 0) {
    if (lane == 0) { c.row_mode[row] = ROW_DEAD; c.row_bias[row] = -INFINITY; c.row_top[row] = -INFINITY; }
    return;
  }
  const float* x = c.logits + (size_t)row * c.V;
  float xv[kSparseMax / 64];
  float lmax = -INFINITY;
#pragma unroll
  for (int k = 0; k < kSparseMax / 64; k++) {
    const int i = lane + 64 * k;
    xv[k] = (i < n) ? x[list[i]] : -INFINITY;
    lmax = fmaxf(lmax, xv[k]);
  }
  const float m = gr_wave_max(lmax);
  double S = 0.0;
  const double rc = -(double)m * ek.c;
  const float lo = m - 600.f;
#pragma unroll
  for (int k = 0; k < kSparseMax / 64; k++)
    if (lane + 64 * k < n) S += exp_rel(fmaxf(xv[k], lo), rc, s_tab, ek);
  S = gr_wave_sum(S);
  const float lse = (float)((double)m + log(S));
  const float bias = __fsub_rn(s_in, lse);
  if (lane == 0) { c.row_bias[row] = bias; c.row_mode[row] = ROW_SPARSE; c.row_top[row] = __fadd_rn(bias, m); }
  keys[lane] = (lmax > -INFINITY) ? __fadd_rn(bias, lmax) : -INFINITY;     // a sparse row has kSparseKeys keys
}

// One launch for both kinds of row: the first n_dense_blocks workgroups stream one row each (those come
// first because they run longest), the rest gather four sparse rows each.  Every row is looked at by
// both kinds; the shared test row_is_sparse decides which of them owns it.
__global__ void __launch_bounds__(kRowThreads) k_rows(SelCtx c, int owns_dead, int n_dense_blocks) {
  if ((int)blockIdx.x < n_dense_blocks) row_dense(c, owns_dead, (int)blockIdx.x);
  else rows_sparse(c, (int)blockIdx.x - n_dense_blocks);
}

// ------------------------------------------------------------------------------------------------
// Per-request selection.
// ------------------------------------------------------------------------------------------------
// Visit every finite candidate of request b.  f(score, flat, pred) is called wave-convergently
// (pred = this lane holds a candidate).  Rows given by bit masks are strided by the whole
// workgroup; rows given by child lists are taken one per wavefront.
template <class F>
__device__ __forceinline__ void for_each_candidate(const SelCtx& c, const MaskView& mv, int b, F&& f) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nw = blockDim.x >> 6;
  if (!c.blob || c.step == 0) {
    for (int w = 0; w < c.W; w++) {
      const int row = b * c.W + w;
      if (c.row_mode[row] == ROW_DEAD) continue;
      const float bias = c.row_bias[row];
      const float* x = c.logits + (size_t)row * c.V;
      const uint32_t flat0 = (uint32_t)w * (uint32_t)c.V;
      for (int v0 = 0; v0 < c.V; v0 += blockDim.x) {
        const int v = v0 + threadIdx.x;
        const bool pred = v < c.V && (!c.blob || ((mv.l0[v >> 5] >> (v & 31)) & 1u));
        f(pred ? __fadd_rn(bias, x[v]) : 0.f, flat0 + v, pred);
      }
    }
  } else {
    for (int w = wave; w < c.W; w += nw) {
      const int row = b * c.W + w;
      if (c.row_mode[row] == ROW_DEAD) continue;
      const float bias = c.row_bias[row];
      const float* x = c.logits + (size_t)row * c.V;
      const uint32_t flat0 = (uint32_t)w * (uint32_t)c.V;
      const int32_t* list;
      int n;
      row_children(c, mv, row, &list, &n);
      for (int i0 = 0; i0 < n; i0 += 64) {
        const int i = i0 + lane;
        const bool pred = i < n;
        const int v = pred ? list[i] : 0;
        f(pred ? __fadd_rn(bias, x[v]) : 0.f, flat0 + v, pred);
      }
    }
  }
}

__device__ __forceinline__ uint64_t composite(float score, uint32_t flat) {
  return ((uint64_t)gr_ordkey(score + 0.0f) << 32) | (uint64_t)(0xffffffffu - flat);     // (+0.0f: -0 and +0 are one score)
}

// Monotone (non-increasing in the score) bin index below the request's best chunk key.
__device__ __forceinline__ int key_bin(float hi, float score) {
  return (int)fminf(fmaxf((hi - score) * 64.0f, 0.f), (float)(kHistBins - 1));
}

// Exact MSB radix select of the W best composite keys over ALL candidates (slow, always correct).
// Leaves the survivors in s_list and returns their number.
__device__ int radix_select_all(const SelCtx& c, const MaskView& mv, int b, uint64_t* s_list, uint32_t* s_hist) {
  __shared__ uint64_t s_prefix;
  __shared__ uint32_t s_need, s_bin, s_cnt;
  __shared__ int s_all;
  const int tid = threadIdx.x, lane = tid & 63;
  uint64_t prefix = 0;       // digits chosen so far (the top 64-shift bits of the W-th largest key)
  uint32_t need = (uint32_t)c.W;
  int shift = 64;            // number of key bits not yet fixed
  bool take_all = false;
  for (int pass = 0; pass < 6; pass++) {
    const int width = (pass < 5) ? 11 : 9;
    const int lo_shift = shift - width;
    const int nbins = 1 << width;
    for (int i = tid; i < nbins; i += kSelThreads) s_hist[i] = 0;
    __syncthreads();
    for_each_candidate(c, mv, b, [&](float score, uint32_t flat, bool pred) {
      const uint64_t k = composite(score, flat);
      const bool in = pred && (pass == 0 || (k >> shift) == prefix);
      const uint32_t dgt = (uint32_t)(k >> lo_shift) & (uint32_t)(nbins - 1);
      // most lanes of a wave usually fall in the same bin on the leading digits: add them as one
      const uint64_t act = __ballot(in);
      if (act) {
        const int leader = __ffsll((unsigned long long)act) - 1;
        const uint32_t d0 = __shfl(dgt, leader, 64);
        const uint64_t same = __ballot(in && dgt == d0);
        if (lane == leader) atomicAdd(&s_hist[d0], (uint32_t)__popcll(same));
        if (in && dgt != d0) atomicAdd(&s_hist[dgt], 1u);
      }
    });
    __syncthreads();
    if (tid < 64) {
      // wave 0: find the bin that holds the need-th largest key
      const int per = nbins / 64;
      uint32_t local = 0;
      for (int i = 0; i < per; i++) local += s_hist[lane * per + i];
      uint32_t incl = local;   // inclusive suffix sum over lanes (higher lane = larger keys)
      for (int o = 1; o < 64; o <<= 1) {
        uint32_t v = __shfl_down(incl, o, 64);
        if (lane + o < 64) incl += v;
      }
      const uint32_t total = __shfl(incl, 0, 64);
      const uint32_t above = incl - local;
      if (total < need) {
        if (lane == 0) s_all = 1;           // fewer candidates than slots: keep them all
      } else if (above < need && need <= incl) {
        uint32_t acc = above;
        int bin = lane * per + per - 1;
        for (;; bin--) {
          const uint32_t h = s_hist[bin];
          if (acc + h >= need) break;
          acc += h;
        }
        s_prefix = (prefix << width) | (uint64_t)bin;
        s_need = need - acc;
        s_bin = s_hist[bin];
        s_all = 0;
      }
    }
    __syncthreads();
    if (s_all) { take_all = true; break; }
    prefix = s_prefix;
    need = s_need;
    shift = lo_shift;
    // everything above the bin (W - need keys) plus the bin itself fits in LDS: stop refining
    if ((uint32_t)c.W - need + s_bin <= (uint32_t)kListCap) break;
  }
  if (tid == 0) s_cnt = 0;
  __syncthreads();
  for_each_candidate(c, mv, b, [&](float score, uint32_t flat, bool pred) {
    const uint64_t k = composite(score, flat);
    if (pred && (take_all || (k >> shift) >= prefix)) {
      const uint32_t idx = atomicAdd(&s_cnt, 1u);
      if (idx < (uint32_t)kListCap) s_list[idx] = k;
    }
  });
  __syncthreads();
  return min((int)s_cnt, kListCap);
}

// Smallest bin t with at least `want` entries in bins 0..t (bin 0 = best scores); the last bin when there are fewer
// than `want` entries in total.  Done by the whole workgroup (every thread owns kHistBins / kSelThreads consecutive
// bins; one scan, one barrier inside): a serial walk by one wavefront over 32 bins per lane costs more than a
// microsecond.  The caller puts a barrier behind it before reading *s_thr.
__device__ __forceinline__ void hist_threshold_all(const uint32_t* s_hist, uint32_t want, int* s_thr, uint32_t* s_redu, int& par) {
  constexpr int per = kHistBins / kSelThreads;
  const int tid = threadIdx.x;
  uint32_t h[per], local = 0;
#pragma unroll
  for (int k = 0; k < per; k++) { h[k] = s_hist[tid * per + k]; local += h[k]; }
  uint32_t total;
  const uint32_t below = block_excl_scan<kSelThreads / 64>(local, &total, s_redu, par);
  if (total < want) {
    if (tid == 0) *s_thr = kHistBins - 1;
  } else if (below < want && want <= below + local) {
    uint32_t acc = below;
    int bin = tid * per;
#pragma unroll
    for (int k = 0; k < per; k++) {
      acc += h[k];
      if (acc >= want) break;
      bin++;
    }
    *s_thr = bin;
  }
}

__global__ void __launch_bounds__(kSelThreads) k_select(SelCtx c) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  uint64_t* s_list = (uint64_t*)smem;
  uint32_t* s_hist = (uint32_t*)(smem + (size_t)kListCap * 8);
  uint32_t* s_chunks = s_hist + kHistBins;
  float* s_rbias = (float*)(s_chunks + kChunkCap);          // per beam row of the request: bias,
  int32_t* s_rmode = (int32_t*)(s_rbias + kMaxW);            // mode,
  int32_t* s_ra = s_rmode + kMaxW;                           // first token (step 1) or table range start (step 2),
  int32_t* s_rb = s_ra + kMaxW;                              // start of the child list (step 1) or table range end (step 2),
  int32_t* s_rc = s_rb + kMaxW;                              // end of the child list (step 1)
  __shared__ float s_redf[kSelThreads / 64];
  __shared__ uint32_t s_redu[2 * (kSelThreads / 64)];
  __shared__ uint16_t s_live[kMaxW];
  int par = 0;
  __shared__ uint32_t s_n, s_nc, s_nlive;
  __shared__ int s_thr;
  const int b = blockIdx.x, tid = threadIdx.x;
  constexpr int NW = kSelThreads / 64;
  MaskView mv;
  if (c.blob) mv = mask_view(c.blob, c.V, c.depth);

  if (tid == 0) { s_n = 0; s_nc = 0; s_nlive = 0; }
  for (int i = tid; i < kHistBins; i += kSelThreads) s_hist[i] = 0;
  __syncthreads();
  // ---- the request's rows: what the rows kernels left, the live ones listed, the best candidate overall
  float hi = -INFINITY;
  for (int w = tid; w < c.W; w += kSelThreads) {
    const size_t row = (size_t)b * c.W + w;
    // (everything a row can need is asked for at once; what a dead row returns is ignored)
    const int mode = c.row_mode[row];
    const float bias = c.row_bias[row], top = c.row_top[row];
    int a = 0, bb = 0, cc = 0;
    if (c.blob && c.step == 1) {
      a = c.prefix_in[row * c.depth];
    } else if (c.blob && c.step == 2) {
      a = c.range_in[2 * row]; bb = c.range_in[2 * row + 1];
    }
    s_rmode[w] = mode;
    s_rbias[w] = bias;
    if (mode != ROW_DEAD) {
      hi = fmaxf(hi, top);
      s_live[atomicAdd(&s_nlive, 1u)] = (uint16_t)w;
      if (c.blob && c.step == 1) {
        // the row's child list, looked up once here for the re-read of gathered chunks and for the output
        const bool ok = mv.ok && a >= 0 && a < c.V;
        bb = ok ? mv.pair_off[a] : 0;
        cc = ok ? mv.pair_off[a + 1] : 0;
      } else if (c.blob && c.step == 2) {
        if (!mv.ok || a < 0 || bb < a || (int64_t)bb > mv.n_items) { a = 0; bb = 0; }
      }
    } else {
      a = 0; bb = 0;
    }
    s_ra[w] = a;
    s_rb[w] = bb;
    s_rc[w] = cc;
  }
  hi = block_max2<NW>(hi, s_redf);         // (has the barriers that publish the row table)
  const int nlive = (int)s_nlive;

  // ---- threshold from the chunk keys of the live rows (the best candidate score of every 1/256th of a
  // streamed row, every 1/64th of a gathered one).  Keys are read once and kept in registers for the
  // second use when they fit (up to 256 live rows).
  const float4* keys4 = (const float4*)(c.chunk_key + (size_t)b * c.W * kChunksPerRow);
  constexpr int KR = 16;                   // float4 of keys per thread held in registers
  const int ngroups = nlive * (kChunksPerRow / 4);
  auto group_of = [&](int idx, int* w, int* g) {           // key group idx -> (row, group in row); false if it holds no keys
    *w = s_live[idx / (kChunksPerRow / 4)];
    *g = idx % (kChunksPerRow / 4);
    return s_rmode[*w] == ROW_DENSE || *g < kSparseKeys / 4;
  };
  int n = 0;
  bool need_fallback = false;
  if (hi > -INFINITY) {
    float4 kq[KR];
#pragma unroll
    for (int i = 0; i < KR; i++) {
      const int idx = tid + i * kSelThreads;
      int w, g;
      kq[i] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
      if (idx < ngroups && group_of(idx, &w, &g)) kq[i] = keys4[(size_t)w * (kChunksPerRow / 4) + g];
    }
    auto bin4 = [&](const float4& k, auto&& f) {
      if (k.x > -INFINITY) f(0, key_bin(hi, k.x));
      if (k.y > -INFINITY) f(1, key_bin(hi, k.y));
      if (k.z > -INFINITY) f(2, key_bin(hi, k.z));
      if (k.w > -INFINITY) f(3, key_bin(hi, k.w));
    };
    uint32_t kb[KR][2];                    // bins of the register-resident keys, 16 bits each (0xffff: no key)
#pragma unroll
    for (int i = 0; i < KR; i++) {
      kb[i][0] = 0xffffffffu; kb[i][1] = 0xffffffffu;
      bin4(kq[i], [&](int j, int bin) {
        atomicAdd(&s_hist[bin], 1u);
        kb[i][j >> 1] = (j & 1) ? ((kb[i][j >> 1] & 0x0000ffffu) | ((uint32_t)bin << 16)) : ((kb[i][j >> 1] & 0xffff0000u) | (uint32_t)bin);
      });
    }
    for (int idx = tid + KR * kSelThreads; idx < ngroups; idx += kSelThreads) {
      int w, g;
      if (group_of(idx, &w, &g)) bin4(keys4[(size_t)w * (kChunksPerRow / 4) + g], [&](int, int bin) { atomicAdd(&s_hist[bin], 1u); });
    }
    __syncthreads();
    hist_threshold_all(s_hist, (uint32_t)c.W, &s_thr, s_redu, par);
    __syncthreads();
    const int thr = s_thr;
    // ---- chunks that reach the threshold
    auto take = [&](int idx, const float4& k) {
      int w, g;
      group_of(idx, &w, &g);
      bin4(k, [&](int j, int bin) {
        if (bin <= thr) {
          const uint32_t pos = atomicAdd(&s_nc, 1u);
          if (pos < (uint32_t)kChunkCap) s_chunks[pos] = ((uint32_t)w << 8) | (uint32_t)(4 * g + j);
        }
      });
    };
#pragma unroll
    for (int i = 0; i < KR; i++) {
      const uint32_t b4[4] = {kb[i][0] & 0xffffu, kb[i][0] >> 16, kb[i][1] & 0xffffu, kb[i][1] >> 16};
      const uint32_t thr_u = (uint32_t)thr;
      if (b4[0] <= thr_u || b4[1] <= thr_u || b4[2] <= thr_u || b4[3] <= thr_u) {      // (0xffff never passes)
        int w, g;
        group_of(tid + i * kSelThreads, &w, &g);
#pragma unroll
        for (int j = 0; j < 4; j++)
          if (b4[j] <= thr_u) {
            const uint32_t pos = atomicAdd(&s_nc, 1u);
            if (pos < (uint32_t)kChunkCap) s_chunks[pos] = ((uint32_t)w << 8) | (uint32_t)(4 * g + j);
          }
      }
    }
    for (int idx = tid + KR * kSelThreads; idx < ngroups; idx += kSelThreads) {
      int w, g;
      if (group_of(idx, &w, &g)) take(idx, keys4[(size_t)w * (kChunksPerRow / 4) + g]);
    }
    __syncthreads();
    const int nc = (int)s_nc;
    if (nc > kChunkCap) {
      need_fallback = true;
    } else {
      // ---- re-read only those chunks; keep their candidates that reach the threshold.  Twelve (chunk, element)
      // slots per thread and round, all of their loads issued before any is used: the usual W-odd chunks of 32
      // elements fit in one round.  bits: 0 = not a candidate, 1 = valid, 2 = valid if in the row's child list.
      const int epc = max(c.epc, kSparseMax / kSparseKeys);
      const int total = nc * epc;
      constexpr int U = 12;
      for (int base = 0; base < total; base += U * kSelThreads) {
        int wv[U], tok[U];
        float x[U];
        uint32_t bits[U];
#pragma unroll
        for (int q = 0; q < U; q++) {
          const int idx = base + q * kSelThreads + tid;
          tok[q] = -1; x[q] = 0.f; bits[q] = 0; wv[q] = 0;
          if (idx < total) {
            const uint32_t ent = s_chunks[idx / epc];
            const int e = idx % epc;
            const int w = (int)(ent >> 8), k = (int)(ent & 255u);
            wv[q] = w;
            const float* xrow = c.logits + ((size_t)b * c.W + w) * c.V;
            if (s_rmode[w] == ROW_DENSE) {
              const int t = (e < c.epc) ? dense_slot_token(c, k, e) : c.V;
              if (t < c.V) {
                tok[q] = t;
                x[q] = xrow[t];
                if (!c.blob) bits[q] = 1u;
                else if (c.step == 0) bits[q] = (mv.l0[t >> 5] >> (t & 31)) & 1u;
                else if (c.step == 1) {
                  const int t1 = s_ra[w];
                  bits[q] = (t1 >= 0 && t1 < c.V) ? ((mv.l1[(size_t)t1 * mv.words + (t >> 5)] >> (t & 31)) & 1u) : 0u;
                } else bits[q] = 2u;
              }
            } else {
              // gathered row: chunk k = children k, k + 64, ...
              const int32_t* list;
              int nlist;
              if (c.step == 1) { list = mv.pair_t2 + s_rb[w]; nlist = s_rc[w] - s_rb[w]; }
              else { list = mv.t3 + s_ra[w]; nlist = s_rb[w] - s_ra[w]; }
              const int i = k + kSparseKeys * e;
              if (k < kSparseKeys && e < kSparseMax / kSparseKeys && i < nlist) {
                const int t = list[i];
                tok[q] = t;
                x[q] = xrow[t];
                bits[q] = 1u;
              }
            }
          }
        }
#pragma unroll
        for (int q = 0; q < U; q++) {
          if (tok[q] < 0 || bits[q] == 0) continue;
          if (bits[q] == 2u) {              // last level, streamed row: membership in the row's short child list
            const int lo = s_ra[wv[q]], nl = s_rb[wv[q]] - lo;
            const int pos = lower_bound_i32(mv.t3 + lo, nl, tok[q]);
            if (!(pos < nl && mv.t3[lo + pos] == tok[q])) continue;
          }
          const float score = __fadd_rn(s_rbias[wv[q]], x[q]);
          if (key_bin(hi, score) <= thr) {
            const uint32_t pos = atomicAdd(&s_n, 1u);
            if (pos < (uint32_t)kListCap) s_list[pos] = composite(score, (uint32_t)wv[q] * (uint32_t)c.V + (uint32_t)tok[q]);
          }
        }
      }
      __syncthreads();
      if (s_n > (uint32_t)kListCap) need_fallback = true;
      n = min((int)s_n, kListCap);
    }
    if (need_fallback) n = radix_select_all(c, mv, b, s_list, s_hist);

    // ---- many survivors (few chunks, or a coarse first threshold): refine on the scores themselves
    if (n > 2 * c.W) {
      uint64_t mine[kListCap / kSelThreads];
      float top = -INFINITY;
#pragma unroll
      for (int k = 0; k < kListCap / kSelThreads; k++) {
        const int i = tid + k * kSelThreads;
        mine[k] = (i < n) ? s_list[i] : 0;
        if (i < n) top = fmaxf(top, gr_ordkey_inv((uint32_t)(mine[k] >> 32)));
      }
      top = block_max2<NW>(top, s_redf);
      for (int i = tid; i < kHistBins; i += kSelThreads) s_hist[i] = 0;
      if (tid == 0) s_n = 0;
      __syncthreads();
#pragma unroll
      for (int k = 0; k < kListCap / kSelThreads; k++)
        if (tid + k * kSelThreads < n) atomicAdd(&s_hist[key_bin(top, gr_ordkey_inv((uint32_t)(mine[k] >> 32)))], 1u);
      __syncthreads();
      hist_threshold_all(s_hist, (uint32_t)c.W, &s_thr, s_redu, par);
      __syncthreads();
      const int thr2 = s_thr;
#pragma unroll
      for (int k = 0; k < kListCap / kSelThreads; k++)
        if (tid + k * kSelThreads < n && key_bin(top, gr_ordkey_inv((uint32_t)(mine[k] >> 32))) <= thr2)
          s_list[atomicAdd(&s_n, 1u)] = mine[k];
      __syncthreads();
      n = (int)s_n;
    }
  }

  // ---- order the survivors (descending composite key = score descending, flat index ascending)
  const uint64_t* s_sorted = s_list;
  if (n > 1 && 2 * n <= kListCap) {
    // Bucket order: histogram bins are ordered by score, so a survivor's place is the number of survivors in
    // better bins plus its rank inside its own (tiny) bin.  Counting sort by bin into the upper half of the list,
    // then every survivor counts the larger keys of its bin.  Exact ties share a bin and are ranked by the key's
    // flat-index half there.
    float top = -INFINITY, bottom = INFINITY;
    for (int i = tid; i < n; i += kSelThreads) { const float sc = gr_ordkey_inv((uint32_t)(s_list[i] >> 32)); top = fmaxf(top, sc); bottom = fminf(bottom, sc); }
    top = block_max2<NW>(top, s_redf);
    bottom = -block_max2<NW>(-bottom, s_redf);
    const float range = top - bottom;
    const float scale = (range > 0.f && range < INFINITY) ? (float)(kHistBins - 1) / range : 0.f;
    auto bin_of = [&](uint64_t key) { return (int)fminf(fmaxf((top - gr_ordkey_inv((uint32_t)(key >> 32))) * scale, 0.f), (float)(kHistBins - 1)); };
    for (int i = tid; i < kHistBins; i += kSelThreads) s_hist[i] = 0;
    __syncthreads();
    for (int i = tid; i < n; i += kSelThreads) atomicAdd(&s_hist[bin_of(s_list[i])], 1u);
    __syncthreads();
    {
      // exclusive prefix over the bins, in place (each thread owns kHistBins / kSelThreads consecutive bins)
      constexpr int per = kHistBins / kSelThreads;
      uint32_t h[per], sum = 0;
#pragma unroll
      for (int k = 0; k < per; k++) { h[k] = s_hist[tid * per + k]; sum += h[k]; }
      uint32_t total;
      uint32_t run = block_excl_scan<NW>(sum, &total, s_redu, par);
#pragma unroll
      for (int k = 0; k < per; k++) { s_hist[tid * per + k] = run; run += h[k]; }
    }
    __syncthreads();
    uint64_t* s_tmp = s_list + kListCap / 2;
    for (int i = tid; i < n; i += kSelThreads) {
      const uint64_t key = s_list[i];
      s_tmp[atomicAdd(&s_hist[bin_of(key)], 1u)] = key;      // the bin's counter now runs to the bin's end
    }
    __syncthreads();
    for (int q = tid; q < n; q += kSelThreads) {
      const uint64_t key = s_tmp[q];
      const int bin = bin_of(key);
      const int s0 = bin ? (int)s_hist[bin - 1] : 0, s1 = (int)s_hist[bin];
      int cnt = 0;
      for (int j = s0; j < s1; j++) cnt += s_tmp[j] > key;
      s_list[s0 + cnt] = key;
    }
    __syncthreads();
  } else if (n > 1) {
    int n2 = 1;
    while (n2 < n) n2 <<= 1;
    for (int i = n + tid; i < n2; i += kSelThreads) s_list[i] = 0;   // 0 sorts after every real key
    __syncthreads();
    for (int k = 2; k <= n2; k <<= 1) {
      for (int j = k >> 1; j > 0; j >>= 1) {
        for (int i = tid; i < n2; i += kSelThreads) {
          const int ixj = i ^ j;
          if (ixj > i) {
            const uint64_t a = s_list[i], bb = s_list[ixj];
            const bool desc = (i & k) == 0;
            if (desc ? (a < bb) : (a > bb)) { s_list[i] = bb; s_list[ixj] = a; }
          }
        }
        __syncthreads();
      }
    }
  }

  // ---- write the new beam state, best first
  for (int j = tid; j < c.W; j += kSelThreads) {
    const size_t o = (size_t)b * c.W + j;
    int32_t* po = c.prefix_out + o * c.depth;
    for (int k = 0; k < c.depth; k++) po[k] = -1;
    int r_lo = 0, r_hi = 0, item = -1;
    if (j < n) {
      const uint64_t key = s_sorted[j];
      const uint32_t flat = 0xffffffffu - (uint32_t)key;
      const int parent = (int)(flat / (uint32_t)c.V), token = (int)(flat % (uint32_t)c.V);
      c.parent_out[o] = parent;
      c.token_out[o] = token;
      c.scores_out[o] = gr_ordkey_inv((uint32_t)(key >> 32));
      const size_t prow = (size_t)b * c.W + parent;
      for (int k = 0; k < c.step; k++) po[k] = c.prefix_in[prow * c.depth + k];
      po[c.step] = token;
      if (c.blob) {
        if (c.step == 0) {
          r_lo = mv.off1[token]; r_hi = mv.off1[token + 1];
        } else if (c.step == 1) {
          const int p0 = s_rb[parent];                       // (the parent's child list, from the row table)
          const int p = p0 + lower_bound_i32(mv.pair_t2 + p0, s_rc[parent] - p0, token);
          r_lo = mv.pair_row[p]; r_hi = mv.pair_row[p + 1];
        } else {
          const int lo = s_ra[parent];
          r_lo = lo + lower_bound_i32(mv.t3 + lo, s_rb[parent] - lo, token);
          r_hi = r_lo + 1;
          item = r_lo;
        }
      }
    } else {
      c.parent_out[o] = -1;
      c.token_out[o] = -1;
      c.scores_out[o] = -INFINITY;
    }
    c.range_out[2 * o] = r_lo;
    c.range_out[2 * o + 1] = r_hi;
    if (c.item_index_out) c.item_index_out[o] = item;
  }
}

}  // namespace

extern "C" size_t gr_beam_select_workspace_bytes(int32_t B, int32_t W, int32_t V, int32_t depth) {
  if (B <= 0 || W <= 0 || V <= 0 || depth <= 0) return 0;
  const size_t rows = (size_t)B * W;
  return 3 * gr_align256(rows * 4) + gr_align256(rows * kChunksPerRow * 4);
}

extern "C" gr_status gr_beam_select(const gr_select_params* p, void* workspace, size_t workspace_bytes, void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  if (!p) return GR_ERR_INVALID_ARG;
  if (p->B <= 0 || p->W <= 0 || p->V <= 0 || p->depth <= 0 || p->step < 0 || p->step >= p->depth) return GR_ERR_INVALID_ARG;
  if (!p->logits || !p->scores_in || !p->parent_out || !p->token_out || !p->scores_out || !p->prefix_out || !p->range_out)
    return GR_ERR_INVALID_ARG;
  if (p->step > 0 && (!p->prefix_in || (p->mask && !p->range_in))) return GR_ERR_INVALID_ARG;
  if (p->prefix_in && p->prefix_in == p->prefix_out) return GR_ERR_INVALID_ARG;
  if (p->range_in && p->range_in == p->range_out) return GR_ERR_INVALID_ARG;
  if (p->depth != 3 || p->W > 2048 || p->V > 32768 || (int64_t)p->W * p->V >= ((int64_t)1 << 31)) return GR_ERR_UNSUPPORTED;
  if ((int64_t)p->B * p->W >= ((int64_t)1 << 31)) return GR_ERR_UNSUPPORTED;
  if (!workspace || ((uintptr_t)workspace & 255)) return GR_ERR_INVALID_ARG;
  if (workspace_bytes < gr_beam_select_workspace_bytes(p->B, p->W, p->V, p->depth)) return GR_ERR_WORKSPACE_TOO_SMALL;

  SelCtx c;
  c.B = p->B; c.W = p->W; c.V = p->V; c.depth = p->depth; c.step = p->step; c.flags = p->flags;
  c.vec4 = (p->V % 4 == 0) && (((uintptr_t)p->logits & 15) == 0);
  c.epc = c.vec4 ? 4 * ((p->V / 4 + kChunksPerRow - 1) / kChunksPerRow) : (p->V + kChunksPerRow - 1) / kChunksPerRow;
  c.blob = (const char*)p->mask;
  c.logits = p->logits; c.scores_in = p->scores_in; c.prefix_in = p->prefix_in; c.range_in = p->range_in;
  c.parent_out = p->parent_out; c.token_out = p->token_out; c.scores_out = p->scores_out;
  c.prefix_out = p->prefix_out; c.range_out = p->range_out; c.item_index_out = p->item_index_out;
  const size_t rows = (size_t)p->B * p->W;
  char* ws = (char*)workspace;
  c.row_bias = (float*)ws;                 ws += gr_align256(rows * 4);
  c.row_mode = (int32_t*)ws;               ws += gr_align256(rows * 4);
  c.row_top = (float*)ws;                  ws += gr_align256(rows * 4);
  c.chunk_key = (float*)ws;

  const bool has_sparse = p->mask && p->step >= 1 && !(p->flags & GR_SELECT_FORCE_DENSE);
  const size_t sparse_blocks = has_sparse ? (rows + kRowThreads / 64 - 1) / (kRowThreads / 64) : 0;
  hipLaunchKernelGGL(k_rows, dim3((unsigned)(rows + sparse_blocks)), dim3(kRowThreads), 0, stream, c, has_sparse ? 0 : 1, (int)rows);
  // more than 64 KB of LDS must be opted into (per device; cheap, so done on every call)
  GR_HIP_TRY(hipFuncSetAttribute((const void*)k_select, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kSelLdsBytes));
  hipLaunchKernelGGL(k_select, dim3(p->B), dim3(kSelThreads), kSelLdsBytes, stream, c);
  GR_HIP_TRY(hipGetLastError());
  return GR_OK;
}

// ------------------------------------------------------------------------------------------------
// gr_beam_select_noalloc: the same item step for callers that cannot allocate or hand in a workspace.
// The kernels' scratch memory (row bias / mode / best score and the chunk keys) lives in a static device
// array; every GPU the library runs on holds its own copy at its own address, obtained once per device.
// ------------------------------------------------------------------------------------------------
namespace {
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
constexpr int kMaxDevices = 64;
__device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
void* g_scratch_ptr[kMaxDevices];          // device address of `scratch` per device (0 = not looked up yet)
}  // namespace

extern "C" size_t gr_beam_select_noalloc_max_workspace_bytes(void) { return kStaticScratchBytes; }

extern "C" gr_status gr_beam_select_noalloc(const gr_select_params* p, void* stream_) {
  if (!p) return GR_ERR_INVALID_ARG;
  if (p->B <= 0 || p->W <= 0 || p->V <= 0 || p->depth <= 0) return GR_ERR_INVALID_ARG;
  if (gr_beam_select_workspace_bytes(p->B, p->W, p->V, p->depth) > kStaticScratchBytes) return GR_ERR_WORKSPACE_TOO_SMALL;
  int dev = -1;
  GR_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return GR_ERR_UNSUPPORTED;
  if (!g_scratch_ptr[dev]) {
    // (the array's name is only a host-side handle: its device address on the current device is asked for once)
    void* ptr = nullptr;
    GR_HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return GR_ERR_HIP;
    g_scratch_ptr[dev] = ptr;
  }
  // nothing in the workspace has to start at zero: every word a call reads is written by that call first
  return gr_beam_select(p, g_scratch_ptr[dev], kStaticScratchBytes, stream_);
}

