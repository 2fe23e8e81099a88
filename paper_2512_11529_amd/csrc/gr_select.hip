// gr_beam_select: beam item step (paper Sections 6.1-6.3) on gfx950, one fused kernel.
//
// k_item       grid = B requests x G workgroups; a workgroup owns kRowsPerWG consecutive beam rows of one
//              request and walks them one after the other:
//                streamed rows (all four wavefronts): validity bits staged in LDS (dense level-0 /
//                  level-1 mask rows, or the row's sparse last-level positions set in an empty mask),
//                  logits read ONCE with 16-byte loads and kept in registers for the max, the fp64
//                  sum-exp and the candidate scan;
//                gathered rows (few valid children), one wavefront each: only those logits are read.
//              Selection never sorts the W*V candidates and never re-reads a logit.  Every workgroup
//              keeps a small pool of candidates in LDS together with a threshold tau that at least W
//              known candidates reach; a row appends only its candidates >= tau (a handful per row once
//              tau has settled), the pool is thinned with a histogram whenever it fills, and tau only
//              rises - the early-termination idea of Section 6.2 (stop looking at anything that can no
//              longer enter the top W) in data-parallel form.  tau is shared between the workgroups of
//              a request through one atomic word.  A finished workgroup publishes its <= W + slack
//              survivors and takes a ticket; the LAST workgroup of a request to arrive merges the
//              published lists, orders the final W exactly (score descending, flat index ascending)
//              and writes the new beam state.  No workgroup ever waits for another.
//              If a pool overflows (tens of thousands of exact ties) the last workgroup falls back to an
//              exact MSB radix select over all candidates of the request.
// k_item_init  clears the per-request control words (ticket, list length, shared tau, overflow flag).
//              k_item leaves them cleared again, so a caller that reuses a workspace may skip it
//              (GR_SELECT_WORKSPACE_CLEAN).
//
// Arithmetic that decides beam order is fixed: m = fp32 max over valid logits, S = fp64 sum of
// exp(x - m), lse = fp32(m + log S), bias = score_in - lse (fp32), cand = bias + x (fp32), with no
// fused multiply-add in the last two operations.
#include "gr_internal.hpp"

namespace {

constexpr int kT = 256;              // threads per workgroup
constexpr int kNW = kT / 64;
constexpr int kMaxRows = 16;         // most beam rows a workgroup walks (the host picks 8..16, see sel_layout)
constexpr int kSparseMax = 256;      // rows with at most this many valid children are gathered, not streamed
constexpr int kHistBins = 1024;
constexpr int kMaxMaskWords = 1024;  // V <= 32768
constexpr int kRegV4 = 8;            // float4 per thread kept in registers (V <= 8192)
constexpr int kQueueMax = kHistBins; // valid logits of a streamed row compacted before exponentiation (shares the histogram's LDS)
constexpr int kMaxW = 2048;
constexpr int kFlushSlack = 256;     // a workgroup publishes at most W + kFlushSlack survivors
constexpr int kCtlWords = 8;         // control words per request
enum { CTL_TICKET = 0, CTL_COUNT = 1, CTL_TAU = 2, CTL_OVERFLOW = 3 };

enum { ROW_DEAD = 0, ROW_DENSE = 1, ROW_SPARSE = 2 };

// Phase timestamps of every workgroup (100 MHz wall clock), debug builds only.
#ifdef GR_TIMELINE
#define GR_TL(c, k) do { if ((c).dbg && threadIdx.x == 0) (c).dbg[(size_t)blockIdx.x * 32 + (k)] = wall_clock64(); } while (0)
#else
#define GR_TL(c, k) do { } while (0)
#endif

struct SelCtx {
#ifdef GR_TIMELINE
  unsigned long long* dbg;
#endif
  int B, W, V, depth, step, flags;
  int vec4;                  // V % 4 == 0 and rows 16-byte aligned
  int R;                     // beam rows per workgroup
  int G;                     // workgroups per request
  int cap;                   // candidates a workgroup's LDS pool holds
  int flush_cap;             // candidates a workgroup may publish
  int words;                 // ceil(V / 32)
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
  uint32_t* ctl;             // workspace [B*kCtlWords]
  uint64_t* list;            // workspace [B][G*flush_cap] published survivors
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

__device__ __forceinline__ MaskView mask_view(const SelCtx& c) {
  const gr_mask_header* h = (const gr_mask_header*)c.blob;
  MaskView m;
  m.l0 = (const uint32_t*)(c.blob + h->off_l0);
  m.l1 = (const uint32_t*)(c.blob + h->off_l1);
  m.off1 = (const int32_t*)(c.blob + h->off_off1);
  m.pair_off = (const int32_t*)(c.blob + h->off_pair_off);
  m.pair_t2 = (const int32_t*)(c.blob + h->off_pair_t2);
  m.pair_row = (const int32_t*)(c.blob + h->off_pair_row);
  m.t3 = (const int32_t*)(c.blob + h->off_t3);
  m.words = h->words;
  m.n_items = h->n_items;
  m.ok = h->magic == GR_MASK_MAGIC && h->V == c.V && h->depth == c.depth;
  return m;
}

// The valid children of a beam row as a sorted token list (steps 1 and 2).  A prefix or range that
// this mask could not have produced yields an empty list instead of an out-of-bounds read.
__device__ __forceinline__ void row_children(const SelCtx& c, const MaskView& mv, int row, const int32_t** list, int* n) {
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

// Does this row get gathered (true) or streamed (false)?
__device__ __forceinline__ bool row_is_sparse(const SelCtx& c, int n_children) {
  return c.blob && c.step >= 1 && !(c.flags & GR_SELECT_FORCE_DENSE) && n_children <= kSparseMax;
}

__device__ __forceinline__ int lower_bound_i32(const int32_t* a, int n, int key) {
  int lo = 0, hi = n;
  while (lo < hi) { int mid = (lo + hi) >> 1; if (a[mid] < key) lo = mid + 1; else hi = mid; }
  return lo;
}

// e^(x - ref) in fp64 for fp32 x <= ref (and not more than ~700 below it), about 1e-14 relative:
//   t = (x - ref) * 512/ln2 = n + f with n = rint(t), |f| <= 1/2, both from one addition of 1.5 * 2^52 (the sum's
//   low word then holds n); e^(x-ref) = 2^(n>>9) * 2^((n&511)/512) * 2^(f/512) with
//   2^(f/512) - 1 = f (c1 + f (c2 + f c3)), c_k = (ln2/512)^k / k!  (truncation < 1e-14), the middle factor from a
//   512-entry table in LDS and the power of two added to the exponent field.  Ten fp64 and four integer operations;
//   all run at the full rate.  The error is far below what the single fp32 rounding of lse = m + log S can see.
// The constants live in scalar registers (set up once per kernel): left to itself the compiler
// re-materialises each 64-bit literal with vector moves next to every use.
constexpr int kExpTab = 512;
struct ExpK { double c, magic, c1, c2, c3; };
__device__ __forceinline__ ExpK exp_consts() {
  constexpr double a = 0x1.62e42fefa39efp-1 / 512.0;            // ln2 / 512
  ExpK k = {512.0 * 0x1.71547652b82fep+0, 0x1.8p+52, a, a * a / 2.0, a * a * a / 6.0};
  asm volatile("" : "+s"(k.c), "+s"(k.magic), "+s"(k.c1), "+s"(k.c2), "+s"(k.c3));
  return k;
}
// The table 2^(j/512), j = 0..511, computed by the workgroup itself (two exp2 per thread).
__device__ __forceinline__ void exp_table_init(double* tab) {
  for (int j = threadIdx.x; j < kExpTab; j += blockDim.x) tab[j] = exp2((double)j * (1.0 / kExpTab));
}
// rc = -(double)ref * k.c; x must be >= ref - 600 (callers clamp: what is cut off is below 1e-260 of the sum)
__device__ __forceinline__ double exp_rel(float x, double rc, const double* tab, const ExpK& k) {
  const double t = fma((double)x, k.c, rc);
  const double u = t + k.magic;
  const int n = __double2loint(u);
  const double f = t - (u - k.magic);
  double p = fma(f, k.c3, k.c2);
  p = fma(p, f, k.c1);
  p = p * f;
  const double tj = tab[n & (kExpTab - 1)];
  const double r = fma(tj, p, tj);
  return __hiloint2double(__double2hiint(r) + ((n >> 9) << 20), __double2loint(r));
}

// max without the NaN-quieting instructions fmaxf() drags in (NaN inputs are outside the contract)
__device__ __forceinline__ float max_raw(float a, float b) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}

__device__ __forceinline__ uint64_t composite(float score, uint32_t flat) {
  return ((uint64_t)gr_ordkey(score + 0.0f) << 32) | (uint64_t)(0xffffffffu - flat);     // (+0.0f: -0 and +0 are one score)
}
__device__ __forceinline__ float key_score(uint64_t key) { return gr_ordkey_inv((uint32_t)(key >> 32)); }

// Monotone (non-increasing in the score) map of the scores in [bottom, top] onto the histogram bins, best score
// in bin 0.  The scale follows the spread of the values at hand, so a wide spread (few valid children per row,
// beams far apart) thins as well as a narrow one.
struct BinMap { float top, scale; };
__device__ __forceinline__ BinMap bin_map(float top, float bottom) {
  const float range = top - bottom;
  BinMap bm = {top, (range > 0.f && range < INFINITY) ? (float)(kHistBins - 1) / range : 0.f};
  return bm;
}
__device__ __forceinline__ int key_bin(const BinMap& bm, float score) {
  return (int)fminf(fmaxf((bm.top - score) * bm.scale, 0.f), (float)(kHistBins - 1));
}

// Data that one workgroup writes and another workgroup of the same launch reads (published survivors, row bias and
// mode) moves with agent-scope relaxed atomics: the stores write through the XCD's L2 to memory and the loads
// bypass it, so no workgroup has to write back and invalidate a whole L2 (what an agent-scope fence does on this
// chip - measured at ~0.1 us per workgroup, serialised, when every workgroup executed one).
template <class T>
__device__ __forceinline__ void st_agent(T* p, T v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
template <class T>
__device__ __forceinline__ T ld_agent(const T* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// LDS of a workgroup
struct Lds {
  uint64_t* pool;      // [cap]
  uint32_t* hist;      // [kHistBins]; also the queue of valid logits (float) of a thinly populated streamed row
  uint32_t* mask;      // [words]
  float* next;         // [kRegV4 * kT * 4] staging area of the next streamed row (register-resident kernels)
  double* tab;         // [kExpTab]
  float* redf;         // [2 * kNW]  two slot sets per kind of reduction, see block_max
  double* redd;        // [2 * kNW]
  uint32_t* redu;      // [2 * kNW]
  mutable int par;     // reductions made so far (same in every thread)
  uint32_t* pn;        // pool length
  int* thr;            // histogram threshold bin
  uint32_t* flag;      // scratch word (overflow seen, last-arrival flag, list base)
};

// Workgroup reductions with ONE barrier each: the per-wavefront partials go to one of two slot sets, used
// alternately (every thread makes the same sequence of calls), so a wavefront that is already writing the
// next reduction's partials cannot disturb a slower one that still reads this one's; the set after that is
// only written behind the next reduction's barrier.
__device__ __forceinline__ float block_max(float v, const Lds& L) {
  v = gr_wave_max(v);
  float* slot = L.redf + (L.par & 1) * kNW;
  L.par++;
  if (gr_lane() == 0) slot[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = slot[0];
#pragma unroll
  for (int i = 1; i < kNW; i++) r = fmaxf(r, slot[i]);
  return r;
}
__device__ __forceinline__ float block_min(float v, const Lds& L) { return -block_max(-v, L); }
__device__ __forceinline__ double block_sum(double v, const Lds& L) {
  v = gr_wave_sum(v);
  double* slot = L.redd + (L.par & 1) * kNW;
  L.par++;
  if (gr_lane() == 0) slot[threadIdx.x >> 6] = v;
  __syncthreads();
  double r = slot[0];
#pragma unroll
  for (int i = 1; i < kNW; i++) r += slot[i];
  return r;
}
// exclusive prefix of v over the workgroup's threads (thread order), and the total
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* total, const Lds& L) {
  const int lane = gr_lane(), wave = threadIdx.x >> 6;
  uint32_t incl = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t t = __shfl_up(incl, o, 64);
    if (lane >= o) incl += t;
  }
  uint32_t* slot = L.redu + (L.par & 1) * kNW;
  L.par++;
  if (lane == 63) slot[wave] = incl;
  __syncthreads();
  uint32_t base = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < kNW; i++) { const uint32_t t = slot[i]; if (i < wave) base += t; tot += t; }
  *total = tot;
  return base + incl - v;
}

// Wave 0 only: smallest bin t with at least `want` entries in bins 0..t (bin 0 = best scores); the
// last bin when there are fewer than `want` entries in total.
__device__ __forceinline__ void hist_threshold(const uint32_t* s_hist, uint32_t want, int* s_thr, uint32_t* s_tot = nullptr) {
  const int lane = threadIdx.x & 63;
  constexpr int per = kHistBins / 64;
  uint32_t local = 0;
  for (int i = 0; i < per; i++) local += s_hist[lane * per + i];
  uint32_t incl = local;   // inclusive prefix sum over lanes
  for (int o = 1; o < 64; o <<= 1) {
    uint32_t v = __shfl_up(incl, o, 64);
    if (lane >= o) incl += v;
  }
  const uint32_t tot = __shfl(incl, 63, 64);
  const uint32_t below = incl - local;
  if (s_tot && lane == 0) *s_tot = tot;
  if (tot < want) {
    if (lane == 0) *s_thr = kHistBins - 1;
  } else if (below < want && want <= incl) {
    uint32_t acc = below;
    int bin = lane * per;
    for (;; bin++) { acc += s_hist[bin]; if (acc >= want) break; }
    *s_thr = bin;
  }
}

__device__ __forceinline__ void pool_push(const SelCtx& c, const Lds& L, uint64_t key) {
  const uint32_t idx = atomicAdd(L.pn, 1u);
  if (idx < (uint32_t)c.cap) L.pool[idx] = key;        // a longer pool is noticed at the next thinning point
}

// Thin the pool to the candidates that can still be among the W best of what this workgroup has seen:
// histogram of the pool's scores below its best one, the bin in which the W-th best falls, everything
// in worse bins dropped.  tau becomes the smallest surviving score once at least W candidates are known:
// a later candidate below tau has W better ones ahead of it.  Called by the whole workgroup.
// Returns false when the pool had overflowed (the request then takes the exact fallback).
constexpr int kThinChunk = 8;                  // pool entries per thread and compaction round
__device__ __forceinline__ bool pool_thin(const SelCtx& c, const Lds& L, float* tau) {
  __syncthreads();
  const uint32_t n_raw = *L.pn;
  if (n_raw > (uint32_t)c.cap) return false;
  const int n = (int)n_raw, tid = threadIdx.x;
  if (n == 0) return true;
  float top = -INFINITY, bottom = INFINITY;
  for (int i = tid; i < n; i += kT) { const float s = key_score(L.pool[i]); top = fmaxf(top, s); bottom = fminf(bottom, s); }
  top = block_max(top, L);
  bottom = block_min(bottom, L);
  const BinMap bm = bin_map(top, bottom);
  for (int i = tid; i < kHistBins; i += kT) L.hist[i] = 0;
  __syncthreads();
  for (int i = tid; i < n; i += kT) atomicAdd(&L.hist[key_bin(bm, key_score(L.pool[i]))], 1u);
  __syncthreads();
  if (tid < 64) hist_threshold(L.hist, (uint32_t)c.W, L.thr);
  if (tid == 0) *L.pn = 0;
  __syncthreads();
  const int thr = *L.thr;
  float low = INFINITY;
  // compaction in place, a slab of kThinChunk * kT entries at a time: a slab is in registers before anything is
  // written, and what is kept lands at or below the slab's own start
  for (int i0 = 0; i0 < n; i0 += kThinChunk * kT) {
    uint64_t e[kThinChunk];
#pragma unroll
    for (int k = 0; k < kThinChunk; k++) { const int i = i0 + k * kT + tid; e[k] = (i < n) ? L.pool[i] : 0; }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kThinChunk; k++)
      if (i0 + k * kT + tid < n) {
        const float s = key_score(e[k]);
        if (key_bin(bm, s) <= thr) { L.pool[atomicAdd(L.pn, 1u)] = e[k]; low = fminf(low, s); }
      }
    __syncthreads();
  }
  low = block_min(low, L);
  if (n >= c.W) *tau = fmaxf(*tau, low);
  return true;
}

// A conservative logit threshold for a row: fadd(bias, x) >= tau implies x >= the value returned.
__device__ __forceinline__ float logit_threshold(float tau, float bias) {
  if (!(tau > -INFINITY)) return -INFINITY;
  const float d = __fsub_rn(tau, bias);
  return d - (fabsf(tau) + fabsf(bias) + fabsf(d)) * 0x1p-21f;
}

// ------------------------------------------------------------------------------------------------
// One streamed row, whole workgroup.  REG: the row (V % 4 == 0, V <= 8192, 16-byte aligned) is read
// once and stays in registers; otherwise it is walked from memory (later passes hit in cache).
// ------------------------------------------------------------------------------------------------
template <bool REG>
__device__ __forceinline__ void dense_row(const SelCtx& c, const MaskView& mv, const Lds& L, const ExpK& ek, int row, int w,
                                          float s_in, const int32_t* list, int n_list, float* tau, bool* overflow) {
  const int tid = threadIdx.x, V = c.V;
  const float* x = c.logits + (size_t)row * V;
  // ---- logits requested first, validity bits staged meanwhile
  float4 xr[REG ? kRegV4 : 1];
  const int nv4 = V >> 2;
  if constexpr (REG) {
#pragma unroll
    for (int i = 0; i < kRegV4; i++) {
      const int p = tid + i * kT;
      xr[i] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
      if (p < nv4) xr[i] = *(const float4*)(x + 4 * (size_t)p);
    }
  }
  const int words = c.words;
  int n_valid_known = -1;                   // number of valid entries when the prefix state tells it
  if (c.blob) {
    if (c.step == 0) {
      for (int i = tid; i < words; i += kT) L.mask[i] = mv.ok ? mv.l0[i] : 0u;
    } else if (c.step == 1) {
      const int t1 = c.prefix_in[(size_t)row * c.depth];
      const bool ok = mv.ok && t1 >= 0 && t1 < V;
      const uint32_t* src = mv.l1 + (size_t)(ok ? t1 : 0) * mv.words;
      for (int i = tid; i < words; i += kT) L.mask[i] = ok ? src[i] : 0u;
      n_valid_known = n_list;
    } else {
      // the last level has no dense mask: set the row's valid positions in an empty one
      for (int i = tid; i < words; i += kT) L.mask[i] = 0u;
      __syncthreads();
      for (int i = tid; i < n_list; i += kT) { const int v = list[i]; atomicOr(&L.mask[v >> 5], 1u << (v & 31)); }
      n_valid_known = n_list;
    }
    __syncthreads();
  }
  // ---- this thread's elements: token 4 * (tid + i * kT) + j in register mode, tid + k * kT otherwise.
  // Invalid entries become -inf: they lose every max, add nothing to the sum and pass no threshold.
  uint32_t vbits = 0xffffffffu;
  if constexpr (REG) {
    if (c.blob) {
      vbits = 0;
#pragma unroll
      for (int i = 0; i < kRegV4; i++) {
        const int p = tid + i * kT;
        if (p < nv4) vbits |= ((L.mask[p >> 3] >> (4 * (p & 7))) & 0xfu) << (4 * i);
      }
#pragma unroll
      for (int i = 0; i < kRegV4; i++) {
        if (!((vbits >> (4 * i)) & 1u)) xr[i].x = -INFINITY;
        if (!((vbits >> (4 * i)) & 2u)) xr[i].y = -INFINITY;
        if (!((vbits >> (4 * i)) & 4u)) xr[i].z = -INFINITY;
        if (!((vbits >> (4 * i)) & 8u)) xr[i].w = -INFINITY;
      }
    }
  }
  auto mem_elem = [&](int v) { return (!c.blob || ((L.mask[v >> 5] >> (v & 31)) & 1u)) ? x[v] : -INFINITY; };
  // f(x, token) over this thread's elements
  auto for_each = [&](auto&& f) {
    if constexpr (REG) {
#pragma unroll
      for (int i = 0; i < kRegV4; i++) {
        const int v = 4 * (tid + i * kT);
        f(xr[i].x, v); f(xr[i].y, v + 1); f(xr[i].z, v + 2); f(xr[i].w, v + 3);
      }
    } else {
      for (int v = tid; v < V; v += kT) f(mem_elem(v), v);
    }
  };

  // the request's shared threshold, one relaxed read for the whole workgroup (any older value is just as valid);
  // published to the other threads by the barriers of the reductions below
  if (tid == 0) *L.flag = __hip_atomic_load(&c.ctl[(size_t)(row / c.W) * kCtlWords + CTL_TAU], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  // ---- m = max over valid logits
  float lmax = -INFINITY;
  if constexpr (REG) {
#pragma unroll
    for (int i = 0; i < kRegV4; i++) lmax = max_raw(max_raw(max_raw(lmax, xr[i].x), max_raw(xr[i].y, xr[i].z)), xr[i].w);
  } else {
    for_each([&](float xv, int) { lmax = fmaxf(lmax, xv); });
  }
  if (w % c.R == 1) GR_TL(c, 21);
  const float m = block_max(lmax, L);
  if (w % c.R == 1) GR_TL(c, 22);
  if (!(m > -INFINITY)) {                   // no valid token at all
    if (tid == 0) { st_agent(&c.row_mode[row], (int32_t)ROW_DEAD); st_agent(&c.row_bias[row], -INFINITY); }
    return;
  }
  // ---- S = sum over valid exp(x - m) in fp64
  const double rc = -(double)m * ek.c;
  const float lo = m - 600.f;
  double S = 0.0;
  if (REG && n_valid_known >= 0 && n_valid_known <= kQueueMax) {
    // thinly populated row: the valid logits are packed into a queue (thread order, so the sum is
    // reproducible) and exponentiated with full lanes
    float* q = (float*)L.hist;
    uint32_t total;
    const uint32_t base = block_excl_scan((uint32_t)__popc(vbits), &total, L);
    uint32_t pos = base;
    if constexpr (REG) {
#pragma unroll
      for (int i = 0; i < kRegV4; i++) {
        if (((vbits >> (4 * i)) & 1u) && pos < (uint32_t)kQueueMax) q[pos++] = xr[i].x;
        if (((vbits >> (4 * i)) & 2u) && pos < (uint32_t)kQueueMax) q[pos++] = xr[i].y;
        if (((vbits >> (4 * i)) & 4u) && pos < (uint32_t)kQueueMax) q[pos++] = xr[i].z;
        if (((vbits >> (4 * i)) & 8u) && pos < (uint32_t)kQueueMax) q[pos++] = xr[i].w;
      }
    }
    __syncthreads();
    const int nq = min((int)total, kQueueMax);
    for (int i = tid; i < nq; i += kT) S += exp_rel(max_raw(q[i], lo), rc, L.tab, ek);
  } else if constexpr (REG) {
#pragma unroll
    for (int i = 0; i < kRegV4; i++) {
      S += exp_rel(max_raw(xr[i].x, lo), rc, L.tab, ek);
      S += exp_rel(max_raw(xr[i].y, lo), rc, L.tab, ek);
      S += exp_rel(max_raw(xr[i].z, lo), rc, L.tab, ek);
      S += exp_rel(max_raw(xr[i].w, lo), rc, L.tab, ek);
      // keep the four exponentials of a load together: hoisting the first halves of all 32 costs a hundred registers
      asm volatile("" : "+v"(S)::"memory");
      __builtin_amdgcn_sched_barrier(0);
    }
  } else {
    for_each([&](float xv, int) { if (xv > -INFINITY) S += exp_rel(fmaxf(xv, lo), rc, L.tab, ek); });
  }
  const uint32_t pn0 = *L.pn;               // pool length before this row (read between barriers: no push is in flight)
  if (w % c.R == 1) GR_TL(c, 23);
  S = block_sum(S, L);
  if (w % c.R == 1) GR_TL(c, 24);
  const float lse = (float)((double)m + log(S));
  const float bias = __fsub_rn(s_in, lse);
  if (tid == 0) { st_agent(&c.row_bias[row], bias); st_agent(&c.row_mode[row], (int32_t)ROW_DENSE); }

  // ---- candidates of the row that can still be among the W best
  const uint32_t flat0 = (uint32_t)w * (uint32_t)V;
  float t = *tau;
  {
    // what other workgroups of this request already know (read by one thread before the reductions above and
    // handed out through LDS: every thread must act on the SAME value, the branches below contain barriers)
    const uint32_t shared = *L.flag;
    if (shared) t = fmaxf(t, gr_ordkey_inv(shared));
    *tau = t;
  }
  bool by_histogram = !(t > -INFINITY);
  if (!by_histogram) {
    const float xt = logit_threshold(t, bias);
    for_each([&](float xv, int v) {
      if (xv >= xt) {
        const float s = __fadd_rn(bias, xv);
        if (s >= t) pool_push(c, L, composite(s, flat0 + (uint32_t)v));
      }
    });
    __syncthreads();
    if (*L.pn > (uint32_t)c.cap) {
      // a threshold far below this row (another workgroup's, or one from much weaker rows) let too much through:
      // take the row's pushes back and bound the row by its own W-th best instead
      __syncthreads();
      if (tid == 0) *L.pn = pn0;
      if ((int)pn0 + c.W + kFlushSlack > c.cap) { if (!pool_thin(c, L, tau)) { *overflow = true; return; } }
      by_histogram = true;
    }
  }
  if (by_histogram) {
    // histogram of this row's own candidates between its worst and its best one; the bin in which its W-th
    // best falls bounds what the row can contribute
    float lmin = INFINITY;
    for_each([&](float xv, int) { if (xv > -INFINITY) lmin = fminf(lmin, xv); });
    const BinMap bm = bin_map(__fadd_rn(bias, m), __fadd_rn(bias, block_min(lmin, L)));
    for (int i = tid; i < kHistBins; i += kT) L.hist[i] = 0;
    __syncthreads();
    for_each([&](float xv, int) { if (xv > -INFINITY) atomicAdd(&L.hist[key_bin(bm, __fadd_rn(bias, xv))], 1u); });
    __syncthreads();
    if (tid < 64) hist_threshold(L.hist, (uint32_t)c.W, L.thr);
    __syncthreads();
    const int thr = *L.thr;
    for_each([&](float xv, int v) {
      if (xv > -INFINITY) {
        const float s = __fadd_rn(bias, xv);
        if (key_bin(bm, s) <= thr && s >= t) pool_push(c, L, composite(s, flat0 + (uint32_t)v));
      }
    });
    __syncthreads();
  }
  const uint32_t pn = *L.pn;
  if (w % c.R == 1) GR_TL(c, 25);
  if (pn > (uint32_t)c.cap) { *overflow = true; return; }
  if ((int)pn >= c.cap / 2 || (!(*tau > -INFINITY) && (int)pn >= c.W)) {
    if (!pool_thin(c, L, tau)) { *overflow = true; return; }
    // let the other workgroups of the request profit at once
    if (tid == 0 && *tau > -INFINITY) atomicMax(&c.ctl[(size_t)(row / c.W) * kCtlWords + CTL_TAU], gr_ordkey(*tau + 0.0f));
  }
}

// ------------------------------------------------------------------------------------------------
// Streamed rows, register-resident form (V % 4 == 0, V <= 8192, rows 16-byte aligned, W <= kT): the workgroup's
// rows are classified by eight threads at once, the NEXT streamed row's logits and mask words are requested
// before the current row is worked on (two register sets), the validity bits come straight from the mask row in
// memory (no LDS staging, no barrier), and a row whose best candidate cannot reach tau costs a thread one compare.
// ------------------------------------------------------------------------------------------------
// The register-resident kernel is compiled once per kind of call (MODE 0: no mask; 1, 2, 3: masked levels 0, 1, 2)
// so that none of them carries the others' branches and pointers; MODE -1 decides at run time.
template <int MODE> __device__ __forceinline__ bool is_masked(const SelCtx& c) { if constexpr (MODE < 0) return c.blob != nullptr; else return MODE != 0; }
template <int MODE> __device__ __forceinline__ int level_of(const SelCtx& c) { if constexpr (MODE <= 0) return c.step; else return MODE - 1; }

struct RowMeta {           // one per row of the workgroup, in LDS
  float s_in;
  int cls;                 // ROW_DEAD / ROW_DENSE / ROW_SPARSE
  int n_list;              // valid children (levels 1, 2), else -1
  int t1;                  // first token of the prefix (level 1), else -1
  const int32_t* list;     // sorted valid children (levels 1, 2)
};
struct RowRegs {
  float4 x[kRegV4];        // tokens 4 * (tid + i * kT) .. + 3
  uint32_t mw[kRegV4];     // the mask words that hold this thread's validity nibbles (levels 0 and 1)
};

// Request the next streamed row: its logits go straight from memory into the workgroup's LDS staging area
// (LDS-direct loads: no registers are tied up while the current row is worked on; lane l of a wavefront's i-th
// load lands at slot (i * kT + tid) * 16 bytes), its mask words into eight registers.
template <int MODE>
__device__ __forceinline__ void row_prefetch(const SelCtx& c, const MaskView& mv, const Lds& L, int row, const RowMeta& rm, uint32_t (&mw)[kRegV4]) {
  const int tid = threadIdx.x, nv4 = c.V >> 2;
  const float* x = c.logits + (size_t)row * c.V;
#pragma unroll
  for (int i = 0; i < kRegV4; i++) {
    const int p = tid + i * kT;
    if (p < nv4)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(x + 4 * (size_t)p),
                                       (__attribute__((address_space(3))) void*)(L.next + (size_t)(i * kT + (tid & ~63)) * 4), 16, 0, 0);
  }
  if (is_masked<MODE>(c)) {
    const int step = level_of<MODE>(c);
    const uint32_t* mrow = nullptr;
    if (step == 0) mrow = mv.ok ? mv.l0 : nullptr;
    else if (step == 1) mrow = (mv.ok && rm.t1 >= 0 && rm.t1 < c.V) ? mv.l1 + (size_t)rm.t1 * mv.words : nullptr;
#pragma unroll
    for (int i = 0; i < kRegV4; i++) {
      const int wi = (tid >> 3) + 32 * i;          // float4 p = tid + i * kT has its nibble in word p >> 3
      mw[i] = (mrow && wi < c.words) ? mrow[wi] : 0u;
    }
  }
}
// Take the staged row into registers (every thread reads back exactly what its own loads brought in).
__device__ __forceinline__ void row_take(const SelCtx& c, const Lds& L, RowRegs& R) {
  const int tid = threadIdx.x, nv4 = c.V >> 2;
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
  for (int i = 0; i < kRegV4; i++) {
    const int p = tid + i * kT;
    const float4 v = *(const float4*)(L.next + (size_t)(i * kT + tid) * 4);
    R.x[i] = (p < nv4) ? v : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
  }
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");      // the staging area may be overwritten by this thread's next request
}

template <int MODE>
__device__ __forceinline__ void row_process(const SelCtx& c, const MaskView& mv, const Lds& L, const ExpK& ek, int row, int w,
                                            const RowMeta& rm, RowRegs& R, uint32_t shared_tau, float* tau, bool* overflow) {
  const int tid = threadIdx.x, V = c.V, nv4 = V >> 2;
  const bool masked = is_masked<MODE>(c);
  const int step = level_of<MODE>(c);
  float4(&xr)[kRegV4] = R.x;
  // ---- validity bits: bit 4 i + j <-> token 4 (tid + i kT) + j.  Invalid entries become -inf: they lose every
  // max, add nothing to the sum and pass no threshold.
  uint32_t vbits = 0;
  if (!masked) {
#pragma unroll
    for (int i = 0; i < kRegV4; i++) if (tid + i * kT < nv4) vbits |= 0xfu << (4 * i);
  } else {
#pragma unroll
    for (int i = 0; i < kRegV4; i++) vbits |= ((R.mw[i] >> (4 * (tid & 7))) & 0xfu) << (4 * i);
    if (step == 2) {
      // the last level has no dense mask: the row's few valid positions are set one by one (Section 6.1's sparse form
      // applied to an existing mask)
      if (rm.n_list <= 64) {
        // (scalar loads: they do not queue up behind the next row's vector loads)
        const int32_t* lp = (const int32_t*)(((uint64_t)__builtin_amdgcn_readfirstlane((int)((uint64_t)rm.list >> 32)) << 32) |
                                             (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(uint64_t)rm.list));
        const int nl = __builtin_amdgcn_readfirstlane(rm.n_list);
        for (int e = 0; e < nl; e++) {
          const int t = lp[e];
          if (((t >> 2) & (kT - 1)) == tid) vbits |= 1u << (4 * (t >> 10) + (t & 3));
        }
      } else {
        for (int i = tid; i < c.words; i += kT) L.mask[i] = 0u;
        __syncthreads();
        for (int i = tid; i < rm.n_list; i += kT) { const int v = rm.list[i]; atomicOr(&L.mask[v >> 5], 1u << (v & 31)); }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < kRegV4; i++) {
          const int p = tid + i * kT;
          if (p < nv4) vbits |= ((L.mask[p >> 3] >> (4 * (p & 7))) & 0xfu) << (4 * i);
        }
        __syncthreads();
      }
    }
#pragma unroll
    for (int i = 0; i < kRegV4; i++) {
      if (!((vbits >> (4 * i)) & 1u)) xr[i].x = -INFINITY;
      if (!((vbits >> (4 * i)) & 2u)) xr[i].y = -INFINITY;
      if (!((vbits >> (4 * i)) & 4u)) xr[i].z = -INFINITY;
      if (!((vbits >> (4 * i)) & 8u)) xr[i].w = -INFINITY;
    }
  }
  // ---- m = max over valid logits
  float lmax = -INFINITY;
#pragma unroll
  for (int i = 0; i < kRegV4; i++) lmax = max_raw(max_raw(max_raw(lmax, xr[i].x), max_raw(xr[i].y, xr[i].z)), xr[i].w);
  if (w % c.R == 1) GR_TL(c, 21);
  const float m = block_max(lmax, L);
  if (w % c.R == 1) GR_TL(c, 22);
  if (!(m > -INFINITY)) {                   // no valid token at all
    if (tid == 0) { st_agent(&c.row_mode[row], (int32_t)ROW_DEAD); st_agent(&c.row_bias[row], -INFINITY); }
    return;
  }
  // ---- S = sum over valid exp(x - m) in fp64
  const double rc = -(double)m * ek.c;
  const float lo = m - 600.f;
  double S = 0.0;
  const uint32_t pn0 = *L.pn;               // pool length before this row (read between barriers: no push is in flight)
  if (masked && step >= 1 && rm.n_list <= kQueueMax) {
    // thinly populated row: the valid logits are packed into a queue (thread order, so the sum is
    // reproducible) and exponentiated with full lanes
    float* q = (float*)L.hist;
    uint32_t total;
    uint32_t pos = block_excl_scan((uint32_t)__popc(vbits), &total, L);
#pragma unroll
    for (int i = 0; i < kRegV4; i++) {
      if (((vbits >> (4 * i)) & 1u) && pos < (uint32_t)kQueueMax) q[pos++] = xr[i].x;
      if (((vbits >> (4 * i)) & 2u) && pos < (uint32_t)kQueueMax) q[pos++] = xr[i].y;
      if (((vbits >> (4 * i)) & 4u) && pos < (uint32_t)kQueueMax) q[pos++] = xr[i].z;
      if (((vbits >> (4 * i)) & 8u) && pos < (uint32_t)kQueueMax) q[pos++] = xr[i].w;
    }
    __syncthreads();
    const int nq = min((int)total, kQueueMax);
    for (int i = tid; i < nq; i += kT) S += exp_rel(max_raw(q[i], lo), rc, L.tab, ek);
  } else {
#pragma unroll
    for (int i = 0; i < kRegV4; i++) {
      S += exp_rel(max_raw(xr[i].x, lo), rc, L.tab, ek);
      S += exp_rel(max_raw(xr[i].y, lo), rc, L.tab, ek);
      S += exp_rel(max_raw(xr[i].z, lo), rc, L.tab, ek);
      S += exp_rel(max_raw(xr[i].w, lo), rc, L.tab, ek);
      // keep the four exponentials of a load together: hoisting the first halves of all 32 costs a hundred registers
      asm volatile("" : "+v"(S)::"memory");
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  if (w % c.R == 1) GR_TL(c, 23);
  S = block_sum(S, L);                      // (its barrier also ends every read of the queue)
  if (w % c.R == 1) GR_TL(c, 24);
  const float lse = (float)((double)m + log(S));
  const float bias = __fsub_rn(rm.s_in, lse);
  if (w % c.R == 1) GR_TL(c, 26);
  if (tid == 0) { st_agent(&c.row_bias[row], bias); st_agent(&c.row_mode[row], (int32_t)ROW_DENSE); }

  // ---- candidates of the row that can still be among the W best
  const uint32_t flat0 = (uint32_t)w * (uint32_t)V;
  float t = *tau;
  if (shared_tau) t = fmaxf(t, gr_ordkey_inv(shared_tau));     // what other workgroups of the request already know
  *tau = t;
  // The scan proper: a thread whose best candidate is below the threshold is done after one compare.  The
  // others note their first two hits without branching (cheap, and no code per element beyond a few selects);
  // the rare thread with more walks its 32 logits again from memory in a compact loop.
  auto scan = [&](float tt) {
    const float xt = fmaxf(logit_threshold(tt, bias), -3.0e38f);      // (finite: a masked entry, -inf, never passes)
    if (lmax >= xt) {
      float h0 = 0.f, h1 = 0.f;
      int k0 = 0, k1 = 0, cnt = 0;
#pragma unroll
      for (int i = 0; i < kRegV4; i++) {
#pragma unroll
        for (int j = 0; j < 4; j++) {
          const float xv = j == 0 ? xr[i].x : j == 1 ? xr[i].y : j == 2 ? xr[i].z : xr[i].w;
          const bool hit = xv >= xt;
          if (hit && cnt == 1) { h1 = xv; k1 = 4 * i + j; }
          if (hit && cnt == 0) { h0 = xv; k0 = 4 * i + j; }
          cnt += hit;
        }
      }
      // element 4 i + j of this thread is token 4 (tid + i kT) + j
      auto token_of = [&](int e) { return 4 * (tid + (e >> 2) * kT) + (e & 3); };
      if (cnt <= 2) {
        if (cnt >= 1) { const float sc = __fadd_rn(bias, h0); if (sc >= tt) pool_push(c, L, composite(sc, flat0 + (uint32_t)token_of(k0))); }
        if (cnt >= 2) { const float sc = __fadd_rn(bias, h1); if (sc >= tt) pool_push(c, L, composite(sc, flat0 + (uint32_t)token_of(k1))); }
      } else {
        const float* xrow = c.logits + (size_t)row * V;
        for (int i = 0; i < kRegV4; i++) {
          const int pp = tid + i * kT;
          if (pp >= nv4) break;
          const float4 v4 = *(const float4*)(xrow + 4 * (size_t)pp);
          const uint32_t nib = vbits >> (4 * i);
          const float e4[4] = {v4.x, v4.y, v4.z, v4.w};
#pragma unroll
          for (int j = 0; j < 4; j++)
            if (((nib >> j) & 1u) && e4[j] >= xt) {
              const float sc = __fadd_rn(bias, e4[j]);
              if (sc >= tt) pool_push(c, L, composite(sc, flat0 + (uint32_t)(4 * pp + j)));
            }
        }
      }
    }
  };
  // Nothing useful is known (or the threshold at hand let far too much through): bound the row by its own W-th
  // best.  Every thread offers its two best valid candidates (2 kT >= 2 W of them); the bin in which the W-th best
  // of those falls gives a score that at least W candidates of this row reach.
  auto row_bound = [&](float t_now) -> float {
    float a1 = -INFINITY, a2 = -INFINITY;
#pragma unroll
    for (int i = 0; i < kRegV4; i++) {
      a2 = max_raw(a2, fminf(a1, xr[i].x)); a1 = max_raw(a1, xr[i].x);
      a2 = max_raw(a2, fminf(a1, xr[i].y)); a1 = max_raw(a1, xr[i].y);
      a2 = max_raw(a2, fminf(a1, xr[i].z)); a1 = max_raw(a1, xr[i].z);
      a2 = max_raw(a2, fminf(a1, xr[i].w)); a1 = max_raw(a1, xr[i].w);
    }
    const float s1 = __fadd_rn(bias, a1), s2 = __fadd_rn(bias, a2);
    const float worst = block_min((a2 > -INFINITY) ? s2 : ((a1 > -INFINITY) ? s1 : INFINITY), L);
    const BinMap bm = bin_map(__fadd_rn(bias, m), worst);
    for (int i = tid; i < kHistBins; i += kT) L.hist[i] = 0;
    __syncthreads();
    if (a1 > -INFINITY) atomicAdd(&L.hist[key_bin(bm, s1)], 1u);
    if (a2 > -INFINITY) atomicAdd(&L.hist[key_bin(bm, s2)], 1u);
    __syncthreads();
    if (tid < 64) hist_threshold(L.hist, (uint32_t)c.W, L.thr, L.flag);
    __syncthreads();
    const int thr = *L.thr;
    const bool enough = *L.flag >= (uint32_t)c.W;
    float low = INFINITY;
    if (a1 > -INFINITY && key_bin(bm, s1) <= thr) low = s1;
    if (a2 > -INFINITY && key_bin(bm, s2) <= thr) low = s2;     // (s2 <= s1)
    low = block_min(low, L);
    return enough ? fmaxf(t_now, low) : t_now;   // fewer than W offers: the row keeps everything tau allows
  };
  bool boot = !(t > -INFINITY);
  if (!boot) {
    scan(t);
    if (w % c.R == 1) GR_TL(c, 27);
    __syncthreads();
    if (*L.pn > (uint32_t)c.cap) {
      // a threshold far below this row (another workgroup's, or one from much weaker rows) let too much through:
      // take the row's pushes back and bound the row by its own W-th best instead
      __syncthreads();
      if (tid == 0) *L.pn = pn0;
      if ((int)pn0 + c.W + kFlushSlack > c.cap) { if (!pool_thin(c, L, tau)) { *overflow = true; return; } }
      t = *tau;
      boot = true;
    }
  }
  if (boot) {
    scan(row_bound(t));
    __syncthreads();
    if (*L.pn > (uint32_t)c.cap) { *overflow = true; return; }
  }
  const uint32_t pn = *L.pn;
  if (w % c.R == 1) GR_TL(c, 25);
  if ((int)pn >= c.cap / 2 || (!(*tau > -INFINITY) && (int)pn >= c.W)) {
    if (!pool_thin(c, L, tau)) { *overflow = true; return; }
    // let the other workgroups of the request profit at once
    if (tid == 0 && *tau > -INFINITY) atomicMax(&c.ctl[(size_t)(row / c.W) * kCtlWords + CTL_TAU], gr_ordkey(*tau + 0.0f));
  }
}

// ------------------------------------------------------------------------------------------------
// One gathered row (at most kSparseMax valid children), one wavefront: only the valid logits are read
// (Section 6.1's sparse form).
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ void sparse_row(const SelCtx& c, const Lds& L, const ExpK& ek, int row, int w, float s_in,
                                           const int32_t* list, int n, float tau) {
  const int lane = gr_lane();
  if (n == 0) {
    if (lane == 0) { st_agent(&c.row_mode[row], (int32_t)ROW_DEAD); st_agent(&c.row_bias[row], -INFINITY); }
    return;
  }
  const float* x = c.logits + (size_t)row * c.V;
  float xv[kSparseMax / 64];
  int tok[kSparseMax / 64];
  float lmax = -INFINITY;
#pragma unroll
  for (int k = 0; k < kSparseMax / 64; k++) {
    const int i = lane + 64 * k;
    tok[k] = (i < n) ? list[i] : -1;
    xv[k] = (i < n) ? x[tok[k]] : -INFINITY;
    lmax = fmaxf(lmax, xv[k]);
  }
  const float m = gr_wave_max(lmax);
  double S = 0.0;
  const double rc = -(double)m * ek.c;
  const float lo = m - 600.f;
#pragma unroll
  for (int k = 0; k < kSparseMax / 64; k++)
    if (lane + 64 * k < n) S += exp_rel(fmaxf(xv[k], lo), rc, L.tab, ek);
  S = gr_wave_sum(S);
  const float lse = (float)((double)m + log(S));
  const float bias = __fsub_rn(s_in, lse);
  if (lane == 0) { st_agent(&c.row_bias[row], bias); st_agent(&c.row_mode[row], (int32_t)ROW_SPARSE); }
  const uint32_t flat0 = (uint32_t)w * (uint32_t)c.V;
#pragma unroll
  for (int k = 0; k < kSparseMax / 64; k++)
    if (lane + 64 * k < n) {
      const float s = __fadd_rn(bias, xv[k]);
      if (!(tau > -INFINITY) || s >= tau) pool_push(c, L, composite(s, flat0 + (uint32_t)tok[k]));
    }
}

// ------------------------------------------------------------------------------------------------
// Exact fallback: MSB radix select of the W best composite keys over ALL candidates of the request
// (slow, always correct; taken only when a pool overflowed).
// ------------------------------------------------------------------------------------------------
// Visit every finite candidate of request b.  f(score, flat, pred) is called wave-convergently
// (pred = this lane holds a candidate).  Rows given by bit masks are strided by the whole
// workgroup; rows given by child lists are taken one per wavefront.
template <class F>
__device__ __forceinline__ void for_each_candidate(const SelCtx& c, const MaskView& mv, int b, F&& f) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if (!c.blob || c.step == 0) {
    for (int w = 0; w < c.W; w++) {
      const int row = b * c.W + w;
      if (ld_agent(&c.row_mode[row]) == ROW_DEAD) continue;
      const float bias = ld_agent(&c.row_bias[row]);
      const float* x = c.logits + (size_t)row * c.V;
      const uint32_t flat0 = (uint32_t)w * (uint32_t)c.V;
      for (int v0 = 0; v0 < c.V; v0 += kT) {
        const int v = v0 + threadIdx.x;
        const bool pred = v < c.V && (!c.blob || ((mv.l0[v >> 5] >> (v & 31)) & 1u));
        f(pred ? __fadd_rn(bias, x[v]) : 0.f, flat0 + v, pred);
      }
    }
  } else {
    for (int w = wave; w < c.W; w += kNW) {
      const int row = b * c.W + w;
      if (ld_agent(&c.row_mode[row]) == ROW_DEAD) continue;
      const float bias = ld_agent(&c.row_bias[row]);
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

// Leaves the survivors (at most cap, at least min(W, number of candidates)) in the pool; returns their number.
__device__ __forceinline__ int radix_select_all(const SelCtx& c, const MaskView& mv, int b, const Lds& L) {
  __shared__ uint64_t s_prefix;
  __shared__ uint32_t s_need, s_bin, s_cnt;
  __shared__ int s_all;
  const int tid = threadIdx.x, lane = tid & 63;
  uint32_t* s_hist = L.hist;
  uint64_t prefix = 0;       // digits chosen so far (the top 64-shift bits of the W-th largest key)
  uint32_t need = (uint32_t)c.W;
  int shift = 64;            // number of key bits not yet fixed
  bool take_all = false;
  for (int pass = 0; pass < 6; pass++) {
    const int width = (pass < 5) ? 11 : 9;
    const int lo_shift = shift - width;
    const int nbins = 1 << width;
    for (int i = tid; i < nbins; i += kT) s_hist[i] = 0;
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
    // everything above the bin (W - need keys) plus the bin itself fits in the pool: stop refining
    if ((uint32_t)c.W - need + s_bin <= (uint32_t)c.cap) break;
  }
  if (tid == 0) s_cnt = 0;
  __syncthreads();
  for_each_candidate(c, mv, b, [&](float score, uint32_t flat, bool pred) {
    const uint64_t k = composite(score, flat);
    if (pred && (take_all || (k >> shift) >= prefix)) {
      const uint32_t idx = atomicAdd(&s_cnt, 1u);
      if (idx < (uint32_t)c.cap) L.pool[idx] = k;
    }
  });
  __syncthreads();
  return min((int)s_cnt, c.cap);
}

// ------------------------------------------------------------------------------------------------
// Last workgroup of a request: merge the published survivors, order the best W exactly, write the
// new beam state, and leave the control words cleared.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ void finalize_request(const SelCtx& c, const MaskView& mv, const Lds& L, int b) {
  const int tid = threadIdx.x;
  uint32_t* ctl = c.ctl + (size_t)b * kCtlWords;
  const uint32_t n_list = __hip_atomic_load(&ctl[CTL_COUNT], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const bool overflow = __hip_atomic_load(&ctl[CTL_OVERFLOW], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0;
  const uint64_t* src = c.list + (size_t)b * c.G * c.flush_cap;
  int n = 0;
  bool fallback = overflow;
  if (!fallback) {
    if (n_list <= (uint32_t)c.cap) {
      for (uint32_t i0 = 0; i0 < n_list; i0 += 8 * kT) {        // eight loads in flight per thread: they bypass the L2
        uint64_t v[8];
#pragma unroll
        for (int u = 0; u < 8; u++) { const uint32_t i = i0 + u * kT + tid; v[u] = (i < n_list) ? ld_agent(&src[i]) : 0; }
#pragma unroll
        for (int u = 0; u < 8; u++) { const uint32_t i = i0 + u * kT + tid; if (i < n_list) L.pool[i] = v[u]; }
      }
      n = (int)n_list;
      if (tid == 0) *L.pn = n_list;
    } else {
      // more published survivors than the pool holds: a histogram over all of them first
      float top = -INFINITY, bottom = INFINITY;
      for (uint32_t i = tid; i < n_list; i += kT) { const float sc = key_score(ld_agent(&src[i])); top = fmaxf(top, sc); bottom = fminf(bottom, sc); }
      top = block_max(top, L);
      bottom = block_min(bottom, L);
      const BinMap bm = bin_map(top, bottom);
      for (int i = tid; i < kHistBins; i += kT) L.hist[i] = 0;
      if (tid == 0) *L.pn = 0;
      __syncthreads();
      for (uint32_t i = tid; i < n_list; i += kT) atomicAdd(&L.hist[key_bin(bm, key_score(ld_agent(&src[i])))], 1u);
      __syncthreads();
      if (tid < 64) hist_threshold(L.hist, (uint32_t)c.W, L.thr);
      __syncthreads();
      const int thr = *L.thr;
      for (uint32_t i = tid; i < n_list; i += kT) {
        const uint64_t k = ld_agent(&src[i]);
        if (key_bin(bm, key_score(k)) <= thr) pool_push(c, L, k);
      }
      __syncthreads();
      if (*L.pn > (uint32_t)c.cap) fallback = true;
      n = (int)min(*L.pn, (uint32_t)c.cap);
    }
  }
  for (int it = 0; it < 3 && !fallback && n > c.W + kFlushSlack; it++) {      // (each round zooms in on what the last one kept)
    float tau = -INFINITY;
    pool_thin(c, L, &tau);
    n = (int)*L.pn;
  }
  if (fallback) n = radix_select_all(c, mv, b, L);
  __syncthreads();
  GR_TL(c, 14);

  // ---- order the survivors (descending composite key = score descending, flat index ascending)
  uint64_t* s_list = L.pool;
  const uint64_t* s_sorted = s_list;
  if (n > 1 && 2 * n <= c.cap) {
    // Bucket order: the histogram bins are already ordered by score, so a survivor's place is the number of
    // survivors in better bins plus its rank inside its own (tiny) bin.  Counting sort by bin into the upper half
    // of the pool, then every survivor counts the larger keys of its bin.  Exact ties land in one bin and are
    // ranked by the key's flat-index half there.
    float top = -INFINITY, bottom = INFINITY;
    for (int i = tid; i < n; i += kT) { const float sc = key_score(s_list[i]); top = fmaxf(top, sc); bottom = fminf(bottom, sc); }
    top = block_max(top, L);
    bottom = block_min(bottom, L);
    const BinMap bm = bin_map(top, bottom);
    for (int i = tid; i < kHistBins; i += kT) L.hist[i] = 0;
    __syncthreads();
    for (int i = tid; i < n; i += kT) atomicAdd(&L.hist[key_bin(bm, key_score(s_list[i]))], 1u);
    __syncthreads();
    {
      // exclusive prefix over the bins, in place (each thread owns kHistBins / kT consecutive bins)
      constexpr int per = kHistBins / kT;
      uint32_t h[per], sum = 0;
#pragma unroll
      for (int k = 0; k < per; k++) { h[k] = L.hist[tid * per + k]; sum += h[k]; }
      uint32_t total;
      uint32_t run = block_excl_scan(sum, &total, L);
#pragma unroll
      for (int k = 0; k < per; k++) { L.hist[tid * per + k] = run; run += h[k]; }
    }
    __syncthreads();
    uint64_t* s_tmp = s_list + c.cap / 2;
    for (int i = tid; i < n; i += kT) {
      const uint64_t key = s_list[i];
      s_tmp[atomicAdd(&L.hist[key_bin(bm, key_score(key))], 1u)] = key;      // the bin's counter now runs to the bin's end
    }
    __syncthreads();
    for (int q = tid; q < n; q += kT) {
      const uint64_t key = s_tmp[q];
      const int bin = key_bin(bm, key_score(key));
      const int s0 = bin ? (int)L.hist[bin - 1] : 0, s1 = (int)L.hist[bin];
      int cnt = 0;
      for (int j = s0; j < s1; j++) cnt += s_tmp[j] > key;
      s_list[s0 + cnt] = key;
    }
    __syncthreads();
  } else if (n > 1) {
    int n2 = 1;
    while (n2 < n) n2 <<= 1;                                 // n <= cap, and cap is a power of two
    for (int i = n + tid; i < n2; i += kT) s_list[i] = 0;    // 0 sorts after every real key
    __syncthreads();
    for (int k = 2; k <= n2; k <<= 1) {
      for (int j = k >> 1; j > 0; j >>= 1) {
        for (int i = tid; i < n2; i += kT) {
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

  GR_TL(c, 15);
  // ---- write the new beam state, best first
  for (int j = tid; j < c.W; j += kT) {
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
      c.scores_out[o] = key_score(key);
      const size_t prow = (size_t)b * c.W + parent;
      for (int k = 0; k < c.step; k++) po[k] = c.prefix_in[prow * c.depth + k];
      po[c.step] = token;
      if (c.blob) {
        if (c.step == 0) {
          r_lo = mv.off1[token]; r_hi = mv.off1[token + 1];
        } else if (c.step == 1) {
          const int32_t* list; int nl;
          row_children(c, mv, (int)prow, &list, &nl);
          const int p = (int)(list - mv.pair_t2) + lower_bound_i32(list, nl, token);
          r_lo = mv.pair_row[p]; r_hi = mv.pair_row[p + 1];
        } else {
          const int32_t* list; int nl;
          row_children(c, mv, (int)prow, &list, &nl);
          r_lo = (int)(list - mv.t3) + lower_bound_i32(list, nl, token);
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
  // the control words are left as the next call expects them
  if (tid < kCtlWords) ctl[tid] = 0;
}

template <bool REG, int MODE>
__global__ void __launch_bounds__(kT) __attribute__((amdgpu_waves_per_eu(3, 8))) k_item(SelCtx c) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  __shared__ float s_redf[2 * kNW];
  __shared__ double s_redd[2 * kNW];
  __shared__ uint32_t s_redu[2 * kNW];
  __shared__ uint32_t s_pn, s_flag;
  __shared__ int s_thr;
  Lds L;
  L.pool = (uint64_t*)smem;
  L.tab = (double*)(smem + (size_t)c.cap * 8);
  L.hist = (uint32_t*)(L.tab + kExpTab);
  L.mask = L.hist + kHistBins;
  L.next = (float*)(L.mask + ((c.words + 3) & ~3));
  L.redf = s_redf; L.redd = s_redd; L.redu = s_redu; L.par = 0; L.pn = &s_pn; L.thr = &s_thr; L.flag = &s_flag;
  const int tid = threadIdx.x, wave = tid >> 6;
  const int b = (int)blockIdx.x / c.G, g = (int)blockIdx.x % c.G;
  exp_table_init(L.tab);
  if (tid == 0) { s_pn = 0; s_flag = 0; }
  const ExpK ek = exp_consts();
  MaskView mv;
  mv.ok = true;
  if (is_masked<MODE>(c)) mv = mask_view(c);
  __syncthreads();

  GR_TL(c, 0);
  const int w0 = g * c.R, w1 = min(c.W, w0 + c.R);
  float tau = -INFINITY;
  bool overflow = false;
  // ---- the workgroup's rows classified by one thread each (their chains of dependent loads run side by side)
  __shared__ RowMeta s_meta[kMaxRows];
  __shared__ uint32_t s_tauw;
  if (tid < w1 - w0) {
    const int row = b * c.W + w0 + tid;
    RowMeta rm;
    rm.s_in = c.scores_in[row];
    rm.cls = ROW_DENSE; rm.n_list = -1; rm.t1 = -1; rm.list = nullptr;
    if (!(rm.s_in > -INFINITY)) {
      rm.cls = ROW_DEAD;
      st_agent(&c.row_mode[row], (int32_t)ROW_DEAD); st_agent(&c.row_bias[row], -INFINITY);
    } else if (is_masked<MODE>(c) && level_of<MODE>(c) >= 1) {
      rm.n_list = 0;
      if (mv.ok) row_children(c, mv, row, &rm.list, &rm.n_list);
      if (level_of<MODE>(c) == 1) rm.t1 = c.prefix_in[(size_t)row * c.depth];
      if (row_is_sparse(c, rm.n_list)) rm.cls = ROW_SPARSE;
    }
    s_meta[tid] = rm;
  }
  __syncthreads();
  uint32_t dense_rows = 0, sparse_rows = 0;
  for (int k = 0; k < w1 - w0; k++) {
    if (s_meta[k].cls == ROW_DENSE) dense_rows |= 1u << k;
    if (s_meta[k].cls == ROW_SPARSE) sparse_rows |= 1u << k;
  }
  // ---- streamed rows first (the whole workgroup on one row).  A workgroup whose pool has overflowed still
  // walks all its rows: the exact fallback needs every row's bias.
  if constexpr (REG) {
    RowRegs cur;
    uint32_t nmw[kRegV4];
#pragma unroll
    for (int i = 0; i < kRegV4; i++) nmw[i] = 0;
    int k = dense_rows ? __ffs(dense_rows) - 1 : -1;
    uint32_t tw = 0;
    if (k >= 0) row_prefetch<MODE>(c, mv, L, b * c.W + w0 + k, s_meta[k], nmw);
    while (k >= 0) {
      dense_rows &= dense_rows - 1;
      const int kn = dense_rows ? __ffs(dense_rows) - 1 : -1;
      row_take(c, L, cur);
      if (k == 1) GR_TL(c, 28);
      if (tid == 0) s_tauw = tw;            // (requested a row ago: any older value of the threshold is just as valid)
      // the request's shared threshold: one relaxed read for the whole workgroup, used by the NEXT row so that
      // nobody waits for it
      if (tid == 0) tw = ld_agent(&c.ctl[(size_t)b * kCtlWords + CTL_TAU]);
#pragma unroll
      for (int i = 0; i < kRegV4; i++) cur.mw[i] = nmw[i];
      if (kn >= 0) row_prefetch<MODE>(c, mv, L, b * c.W + w0 + kn, s_meta[kn], nmw);
      if (k == 1) GR_TL(c, 29);
      __syncthreads();
      if (k == 1) GR_TL(c, 30);
      const uint32_t shared_tau = s_tauw;
      row_process<MODE>(c, mv, L, ek, b * c.W + w0 + k, w0 + k, s_meta[k], cur, shared_tau, &tau, &overflow);
      if (k < 8) GR_TL(c, 1 + k);
      __syncthreads();                      // (s_tauw is rewritten for the next row)
      k = kn;
    }
  } else {
    while (dense_rows) {
      const int k = __ffs(dense_rows) - 1;
      dense_rows &= dense_rows - 1;
      const RowMeta rm = s_meta[k];
      dense_row<false>(c, mv, L, ek, b * c.W + w0 + k, w0 + k, rm.s_in, rm.list, max(rm.n_list, 0), &tau, &overflow);
      if (k < 8) GR_TL(c, 1 + k);
    }
  }
  GR_TL(c, 9);
  // ---- gathered rows, one per wavefront, kNW at a time
  while (sparse_rows) {
    // the wave-th set bit of the next kNW (fewer while no threshold exists: such a row pushes all its children)
    uint32_t bits = sparse_rows;
    int mine = -1;
    const int room = (c.cap - (int)min(s_pn, (uint32_t)c.cap)) / kSparseMax;
    const int per_round = (tau > -INFINITY) ? kNW : max(1, min(kNW, room));
    for (int k = 0; k < per_round && bits; k++) {
      const int i = __ffs(bits) - 1;
      bits &= bits - 1;
      if (k == wave) mine = i;
    }
    sparse_rows = bits;
    if (mine >= 0) {
      const int w = w0 + mine, row = b * c.W + w;
      sparse_row(c, L, ek, row, w, s_meta[mine].s_in, s_meta[mine].list, s_meta[mine].n_list, tau);
    }
    __syncthreads();
    const uint32_t pn = s_pn;
    __syncthreads();                        // (a fast wavefront's next row must not push before every thread has read pn)
    if (pn > (uint32_t)c.cap) overflow = true;
    else if ((int)pn >= c.cap / 2 || (!(tau > -INFINITY) && (int)pn >= c.W)) {
      if (!pool_thin(c, L, &tau)) overflow = true;
      else if (tid == 0 && tau > -INFINITY) atomicMax(&c.ctl[(size_t)b * kCtlWords + CTL_TAU], gr_ordkey(tau + 0.0f));
    }
  }
  // ---- publish what can still win
  __syncthreads();
  GR_TL(c, 10);
  uint32_t* ctl = c.ctl + (size_t)b * kCtlWords;
  for (int it = 0; it < 3 && !overflow && (int)s_pn > (it ? c.flush_cap : c.W); it++) {      // (each round zooms in on what the last one kept)
    if (!pool_thin(c, L, &tau)) overflow = true;
    __syncthreads();
  }
  __syncthreads();
  uint32_t n_pub = 0;
  if (!overflow) {
    // drop what another workgroup's threshold has already ruled out (one read, handed out through LDS)
    if (tid == 0) s_flag = __hip_atomic_load(&ctl[CTL_TAU], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    const uint32_t shared = s_flag;
    __syncthreads();
    const uint32_t mine_key = (tau > -INFINITY) ? gr_ordkey(tau + 0.0f) : 0u;
    const uint32_t floor_key = max(shared, mine_key);
    const int n = (int)s_pn;
    // count, reserve, write (thread order does not matter: the last workgroup orders by key)
    uint32_t keep = 0;
    for (int i = tid; i < n; i += kT) keep += (uint32_t)(L.pool[i] >> 32) >= floor_key;
    uint32_t total;
    uint32_t pos = block_excl_scan(keep, &total, L);
    if (total > (uint32_t)c.flush_cap) {
      overflow = true;
    } else {
      if (tid == 0) {
        s_flag = total ? atomicAdd(&ctl[CTL_COUNT], total) : 0u;
        if (mine_key > shared) atomicMax(&ctl[CTL_TAU], mine_key);
      }
      __syncthreads();
      uint64_t* dst = c.list + (size_t)b * c.G * c.flush_cap + s_flag;
      for (int i = tid; i < n; i += kT) {
        const uint64_t k = L.pool[i];
        if ((uint32_t)(k >> 32) >= floor_key) st_agent(&dst[pos++], k);
      }
      n_pub = total;
    }
  }
  (void)n_pub;
  if (overflow && tid == 0) atomicOr(&ctl[CTL_OVERFLOW], 1u);
  // ---- ticket: the last workgroup of the request to get here finishes the request.  Every thread first waits
  // until its write-through stores have been acknowledged; the barrier then orders them before the ticket.
  GR_TL(c, 11);
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  __syncthreads();
  GR_TL(c, 12);
  if (tid == 0) s_flag = (atomicAdd(&ctl[CTL_TICKET], 1u) == (uint32_t)c.G - 1u) ? 1u : 0u;
  __syncthreads();
  GR_TL(c, 13);
  if (!s_flag) return;
  if (tid == 0) s_pn = 0;
  __syncthreads();
  {
    // The parameters are read again from the kernel-argument segment (this kernel's only argument sits at its
    // start) through a pointer the compiler cannot see through: the dozen output pointers that only this last step
    // needs would otherwise sit in scalar registers during the whole row loop.
    const SelCtx* cp = (const SelCtx*)__builtin_amdgcn_kernarg_segment_ptr();
    asm volatile("" : "+s"(cp));
    const SelCtx cf = *cp;
    MaskView mvf;
    mvf.ok = true;
    if (cf.blob) mvf = mask_view(cf);
    finalize_request(cf, mvf, L, b);
  }
  GR_TL(c, 20);
}

__global__ void __launch_bounds__(256) k_item_init(uint32_t* ctl, int n) {
  const int i = (int)blockIdx.x * 256 + (int)threadIdx.x;
  if (i < n) ctl[i] = 0;
}

// Room for a thinned pool (about W) plus everything one row may add after being bounded by its own W-th best
// (about W again) plus slack.
int pool_cap(int W) {
  int cap = 1024;
  while (cap < 2 * W + 2 * kFlushSlack) cap <<= 1;
  return cap;
}

// Rows per workgroup: 8, unless a few more (up to kMaxRows) let ALL workgroups of the launch be resident at once
// (3 per CU x 256 CUs): a launch that needs a second round of workgroups pays a whole workgroup lifetime for it.
int rows_per_wg(int B, int W) {
  constexpr int kResident = 3 * 256;
  for (int r = 8; r <= kMaxRows; r++)
    if ((int64_t)B * ((W + r - 1) / r) <= kResident) return r;
  return 8;
}
struct SelLayout { size_t off_bias, off_mode, off_ctl, off_list, total; int R, G, cap, flush_cap; };
SelLayout sel_layout(int B, int W) {
  SelLayout l;
  const size_t rows = (size_t)B * W;
  l.R = rows_per_wg(B, W);
  l.G = (W + l.R - 1) / l.R;
  l.cap = pool_cap(W);
  l.flush_cap = W + kFlushSlack;
  size_t o = 0;
  l.off_ctl = o;  o += gr_align256((size_t)B * kCtlWords * 4);
  l.off_bias = o; o += gr_align256(rows * 4);
  l.off_mode = o; o += gr_align256(rows * 4);
  l.off_list = o; o += gr_align256((size_t)B * l.G * l.flush_cap * 8);
  l.total = o;
  return l;
}

}  // namespace

#ifdef GR_TIMELINE
static unsigned long long* g_timeline = nullptr;
extern "C" void gr_debug_set_timeline(void* p) { g_timeline = (unsigned long long*)p; }
#endif

extern "C" size_t gr_beam_select_workspace_bytes(int32_t B, int32_t W, int32_t V, int32_t depth) {
  if (B <= 0 || W <= 0 || V <= 0 || depth <= 0) return 0;
  return sel_layout(B, W).total;
}

gr_status gr_select_launch(const gr_select_params* p, void* workspace, size_t workspace_bytes, hipStream_t stream) {
  if (!p) return GR_ERR_INVALID_ARG;
  if (p->B <= 0 || p->W <= 0 || p->V <= 0 || p->depth <= 0 || p->step < 0 || p->step >= p->depth) return GR_ERR_INVALID_ARG;
  if (!p->logits || !p->scores_in || !p->parent_out || !p->token_out || !p->scores_out || !p->prefix_out || !p->range_out)
    return GR_ERR_INVALID_ARG;
  if (p->step > 0 && (!p->prefix_in || (p->mask && !p->range_in))) return GR_ERR_INVALID_ARG;
  if (p->prefix_in && p->prefix_in == p->prefix_out) return GR_ERR_INVALID_ARG;
  if (p->range_in && p->range_in == p->range_out) return GR_ERR_INVALID_ARG;
  if (p->depth != 3 || p->W > kMaxW || p->V > 32768 || (int64_t)p->W * p->V >= ((int64_t)1 << 31)) return GR_ERR_UNSUPPORTED;
  if ((int64_t)p->B * p->W >= ((int64_t)1 << 31)) return GR_ERR_UNSUPPORTED;
  if (!workspace || ((uintptr_t)workspace & 255)) return GR_ERR_INVALID_ARG;
  const SelLayout lay = sel_layout(p->B, p->W);
  if ((int64_t)p->B * lay.G >= ((int64_t)1 << 31)) return GR_ERR_UNSUPPORTED;
  if (workspace_bytes < lay.total) return GR_ERR_WORKSPACE_TOO_SMALL;

  SelCtx c;
#ifdef GR_TIMELINE
  c.dbg = g_timeline;
#endif
  c.B = p->B; c.W = p->W; c.V = p->V; c.depth = p->depth; c.step = p->step; c.flags = p->flags;
  c.vec4 = (p->V % 4 == 0) && (((uintptr_t)p->logits & 15) == 0);
  c.R = lay.R; c.G = lay.G; c.cap = lay.cap; c.flush_cap = lay.flush_cap;
  c.words = (p->V + 31) / 32;
  c.blob = (const char*)p->mask;
  c.logits = p->logits; c.scores_in = p->scores_in; c.prefix_in = p->prefix_in; c.range_in = p->range_in;
  c.parent_out = p->parent_out; c.token_out = p->token_out; c.scores_out = p->scores_out;
  c.prefix_out = p->prefix_out; c.range_out = p->range_out; c.item_index_out = p->item_index_out;
  char* ws = (char*)workspace;
  c.ctl = (uint32_t*)(ws + lay.off_ctl);
  c.row_bias = (float*)(ws + lay.off_bias);
  c.row_mode = (int32_t*)(ws + lay.off_mode);
  c.list = (uint64_t*)(ws + lay.off_list);

  if (!(p->flags & GR_SELECT_WORKSPACE_CLEAN)) {
    const int n = p->B * kCtlWords;
    hipLaunchKernelGGL(k_item_init, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, c.ctl, n);
  }
  const bool reg = c.vec4 && p->V <= kRegV4 * 4 * kT && p->W <= kT;
  const size_t lds = (size_t)c.cap * 8 + (size_t)kExpTab * 8 + (size_t)kHistBins * 4 + (size_t)((c.words + 3) & ~3) * 4 +
                     (reg ? (size_t)kRegV4 * kT * 16 : 0);
  const unsigned grid = (unsigned)((int64_t)p->B * lay.G);
  const int mode = !reg ? -1 : (!p->mask ? 0 : 1 + p->step);
#define GR_LAUNCH_ITEM(REG_, MODE_)                                                                                          \
  do {                                                                                                                      \
    if (lds > 64 * 1024)                                                                                                    \
      GR_HIP_TRY(hipFuncSetAttribute((const void*)k_item<REG_, MODE_>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)); \
    hipLaunchKernelGGL((k_item<REG_, MODE_>), dim3(grid), dim3(kT), lds, stream, c);                                        \
  } while (0)
  switch (mode) {
    case 0: GR_LAUNCH_ITEM(true, 0); break;
    case 1: GR_LAUNCH_ITEM(true, 1); break;
    case 2: GR_LAUNCH_ITEM(true, 2); break;
    case 3: GR_LAUNCH_ITEM(true, 3); break;
    default: GR_LAUNCH_ITEM(false, -1); break;
  }
#undef GR_LAUNCH_ITEM
  GR_HIP_TRY(hipGetLastError());
  return GR_OK;
}

extern "C" gr_status gr_beam_select(const gr_select_params* p, void* workspace, size_t workspace_bytes, void* stream_) {
  return gr_select_launch(p, workspace, workspace_bytes, (hipStream_t)stream_);
}
