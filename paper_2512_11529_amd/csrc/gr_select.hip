// gr_beam_select: beam item step (paper Sections 6.1-6.3) on gfx950.
//
// Two kernels per call, no host synchronisation, no allocation:
//   k_row_stats     one workgroup per beam row: valid set from the mask blob, max / fp64 sum-exp over
//                   valid tokens, lse and the row's additive bias (score_in - lse).
//   k_select        one workgroup per request: exact top-W of the request's candidates by
//                   (score descending, flat index ascending) using an MSB radix select on a 64-bit
//                   composite key that stops as soon as the survivors fit in LDS, then a bitonic sort
//                   of the survivors and the write-out of the new beam state.
//
// Arithmetic that decides beam order is fixed: m = fp32 max over valid logits, S = fp64 sum of
// exp(x - m), lse = fp32(m + log S), bias = score_in - lse (fp32), cand = bias + x (fp32), with no
// fused multiply-add in the last two operations.
#include "gr_internal.hpp"

namespace {

constexpr int kRowThreads = 256;
constexpr int kSelThreads = 1024;
constexpr int kSparseMax = 256;     // rows with at most this many valid children are gathered, not streamed
constexpr int kListCap = 4096;      // survivors that fit in LDS
constexpr int kMaxMaskWords = 1024; // V <= 32768

struct SelCtx {
  int B, W, V, depth, step, flags;
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
  int32_t* row_live;         // workspace [B*W]
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
};

__device__ __forceinline__ MaskView mask_view(const char* blob) {
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

// ------------------------------------------------------------------------------------------------
// Kernel 1: per-row statistics.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ float block_max(float v, float* s_red) {
  v = gr_wave_max(v);
  const int wave = threadIdx.x >> 6;
  __syncthreads();
  if (gr_lane() == 0) s_red[wave] = v;
  __syncthreads();
  float r = s_red[0];
  for (int i = 1; i < (int)(blockDim.x >> 6); i++) r = fmaxf(r, s_red[i]);
  return r;
}
__device__ __forceinline__ double block_sum(double v, double* s_red) {
  v = gr_wave_sum(v);
  const int wave = threadIdx.x >> 6;
  __syncthreads();
  if (gr_lane() == 0) s_red[wave] = v;
  __syncthreads();
  double r = s_red[0];
  for (int i = 1; i < (int)(blockDim.x >> 6); i++) r += s_red[i];
  return r;
}

__global__ void __launch_bounds__(kRowThreads) k_row_stats(SelCtx c) {
  __shared__ uint32_t s_mask[kMaxMaskWords];
  __shared__ float s_redf[kRowThreads / 64];
  __shared__ double s_redd[kRowThreads / 64];
  const int row = blockIdx.x;
  const int tid = threadIdx.x;
  const float s_in = c.scores_in[row];
  if (!(s_in > -INFINITY)) {
    if (tid == 0) { c.row_live[row] = 0; c.row_bias[row] = -INFINITY; }
    return;
  }
  const float* x = c.logits + (size_t)row * c.V;
  const int V = c.V;
  const bool force_dense = (c.flags & GR_SELECT_FORCE_DENSE) != 0;

  const int32_t* list = nullptr;
  int n_list = 0;
  bool sparse = false;
  MaskView mv;
  if (c.blob) {
    mv = mask_view(c.blob);
    if (c.step >= 1) {
      row_children(c, mv, row, &list, &n_list);
      sparse = !force_dense && n_list <= kSparseMax;
    }
  }

  float m = -INFINITY;
  double S = 0.0;
  if (sparse) {
    // gather only the valid logits (the sparse mask form of Section 6.1)
    for (int i = tid; i < n_list; i += kRowThreads) m = fmaxf(m, x[list[i]]);
    m = block_max(m, s_redf);
    if (m > -INFINITY)
      for (int i = tid; i < n_list; i += kRowThreads) S += exp((double)x[list[i]] - (double)m);
  } else {
    // dense: a V-bit validity row in LDS, then stream the logits
    const int words = (V + 31) >> 5;
    if (!c.blob) {
      for (int i = tid; i < words; i += kRowThreads) s_mask[i] = 0xffffffffu;
    } else if (c.step == 0) {
      for (int i = tid; i < words; i += kRowThreads) s_mask[i] = mv.l0[i];
    } else if (c.step == 1) {
      const int t1 = c.prefix_in[(size_t)row * c.depth];
      const bool ok = t1 >= 0 && t1 < V;
      const uint32_t* src = mv.l1 + (size_t)(ok ? t1 : 0) * mv.words;
      for (int i = tid; i < words; i += kRowThreads) s_mask[i] = ok ? src[i] : 0u;
    } else {
      // last level has no dense mask: set the row's few valid positions in an empty mask
      for (int i = tid; i < words; i += kRowThreads) s_mask[i] = 0u;
      __syncthreads();
      for (int i = tid; i < n_list; i += kRowThreads) { const int v = list[i]; atomicOr(&s_mask[v >> 5], 1u << (v & 31)); }
    }
    __syncthreads();
    for (int v = tid; v < V; v += kRowThreads)
      if ((s_mask[v >> 5] >> (v & 31)) & 1u) m = fmaxf(m, x[v]);
    m = block_max(m, s_redf);
    if (m > -INFINITY)
      for (int v = tid; v < V; v += kRowThreads)
        if ((s_mask[v >> 5] >> (v & 31)) & 1u) S += exp((double)x[v] - (double)m);
  }
  if (!(m > -INFINITY)) {
    if (tid == 0) { c.row_live[row] = 0; c.row_bias[row] = -INFINITY; }
    return;
  }
  S = block_sum(S, s_redd);
  if (tid == 0) {
    const float lse = (float)((double)m + log(S));
    c.row_bias[row] = __fsub_rn(s_in, lse);
    c.row_live[row] = 1;
  }
}

// ------------------------------------------------------------------------------------------------
// Kernel 2: exact top-W per request.
// ------------------------------------------------------------------------------------------------
// Visit every finite candidate of request b: f(score, flat, pred) is called wave-convergently
// (pred = this lane holds a candidate).
template <class F>
__device__ __forceinline__ void for_each_candidate(const SelCtx& c, const MaskView& mv, int b, F&& f) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nw = blockDim.x >> 6;
  for (int w = wave; w < c.W; w += nw) {
    const int row = b * c.W + w;
    if (!c.row_live[row]) continue;
    const float bias = c.row_bias[row];
    const float* x = c.logits + (size_t)row * c.V;
    const uint32_t flat0 = (uint32_t)w * (uint32_t)c.V;
    if (!c.blob) {
      for (int v0 = 0; v0 < c.V; v0 += 64) {
        const int v = v0 + lane;
        const bool pred = v < c.V;
        f(pred ? __fadd_rn(bias, x[v]) : 0.f, flat0 + v, pred);
      }
    } else if (c.step == 0) {
      for (int v0 = 0; v0 < c.V; v0 += 64) {
        const int v = v0 + lane;
        const bool pred = v < c.V && ((mv.l0[v >> 5] >> (v & 31)) & 1u);
        f(pred ? __fadd_rn(bias, x[v]) : 0.f, flat0 + v, pred);
      }
    } else {
      const int32_t* list; int n;
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
  return ((uint64_t)gr_ordkey(score) << 32) | (uint64_t)(0xffffffffu - flat);
}

__device__ __forceinline__ int lower_bound_i32(const int32_t* a, int n, int key) {
  int lo = 0, hi = n;
  while (lo < hi) { int mid = (lo + hi) >> 1; if (a[mid] < key) lo = mid + 1; else hi = mid; }
  return lo;
}

__global__ void __launch_bounds__(kSelThreads) k_select(SelCtx c) {
  __shared__ uint32_t s_hist[2048];
  __shared__ uint64_t s_list[kListCap];
  __shared__ uint64_t s_prefix;
  __shared__ uint32_t s_need, s_bin, s_cnt;
  __shared__ int s_all;
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
  MaskView mv;
  if (c.blob) mv = mask_view(c.blob);

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
  const int n = min((int)s_cnt, kListCap);
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

  // write the new beam state, best first
  for (int j = tid; j < c.W; j += kSelThreads) {
    const size_t o = (size_t)b * c.W + j;
    int32_t* po = c.prefix_out + o * c.depth;
    for (int k = 0; k < c.depth; k++) po[k] = -1;
    int r_lo = 0, r_hi = 0, item = -1;
    if (j < n) {
      const uint64_t key = s_list[j];
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
}

}  // namespace

extern "C" size_t gr_beam_select_workspace_bytes(int32_t B, int32_t W, int32_t V, int32_t depth) {
  if (B <= 0 || W <= 0 || V <= 0 || depth <= 0) return 0;
  return 2 * gr_align256((size_t)B * W * 4);
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
  c.blob = (const char*)p->mask;
  c.logits = p->logits; c.scores_in = p->scores_in; c.prefix_in = p->prefix_in; c.range_in = p->range_in;
  c.parent_out = p->parent_out; c.token_out = p->token_out; c.scores_out = p->scores_out;
  c.prefix_out = p->prefix_out; c.range_out = p->range_out; c.item_index_out = p->item_index_out;
  c.row_bias = (float*)workspace;
  c.row_live = (int32_t*)((char*)workspace + gr_align256((size_t)p->B * p->W * 4));

  hipLaunchKernelGGL(k_row_stats, dim3(p->B * p->W), dim3(kRowThreads), 0, stream, c);
  hipLaunchKernelGGL(k_select, dim3(p->B), dim3(kSelThreads), 0, stream, c);
  GR_HIP_TRY(hipGetLastError());
  return GR_OK;
}
