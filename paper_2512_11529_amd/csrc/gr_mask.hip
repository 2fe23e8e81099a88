// gr_item_mask_build: valid-item mask blob from the sorted item table (paper Section 6.1).
//
// The table is scanned once.  A row that starts a new first token contributes a level-0 bit and the
// row offsets of that token; a row that starts a new (t1,t2) pair contributes a level-1 bit and one
// entry of the sparse pair list (the CSR form of level 1, which is also the row index of level 2).
// Pair positions come from a three-kernel exclusive scan (block counts, scan of counts, scatter).
#include "gr_internal.hpp"

namespace {

constexpr int kBuildThreads = 256;
constexpr int kRowsPerThread = 8;
constexpr int kRowsPerBlock = kBuildThreads * kRowsPerThread;

__global__ void k_fill_u32(uint32_t* p, size_t n, uint32_t v) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = v;
}

__device__ __forceinline__ bool row_ok_and_flags(const int32_t* items, int64_t i, int V, bool* new_t1, bool* new_pair) {
  const int32_t a = items[3 * i], b = items[3 * i + 1], c = items[3 * i + 2];
  bool ok = (a >= 0 && a < V && b >= 0 && b < V && c >= 0 && c < V);
  if (i == 0) { *new_t1 = true; *new_pair = true; return ok; }
  const int32_t pa = items[3 * i - 3], pb = items[3 * i - 2], pc = items[3 * i - 1];
  // strictly increasing lexicographic order
  bool gt = (a > pa) || (a == pa && (b > pb || (b == pb && c > pc)));
  *new_t1 = (a != pa);
  *new_pair = (a != pa) || (b != pb);
  return ok && gt;
}

// pass 1: validate rows, count pair starts per block
__global__ void __launch_bounds__(kBuildThreads) k_mask_count(const int32_t* items, int64_t n, int V, int32_t* block_counts, int32_t* err) {
  __shared__ int s_cnt;
  if (threadIdx.x == 0) s_cnt = 0;
  __syncthreads();
  int64_t base = (int64_t)blockIdx.x * kRowsPerBlock;
  int cnt = 0;
  bool bad = false;
  for (int k = 0; k < kRowsPerThread; k++) {
    int64_t i = base + (int64_t)k * kBuildThreads + threadIdx.x;
    if (i < n) {
      bool t1, pr;
      if (!row_ok_and_flags(items, i, V, &t1, &pr)) bad = true;
      cnt += pr ? 1 : 0;
    }
  }
  if (bad) atomicOr(err, 1);
  atomicAdd(&s_cnt, cnt);
  __syncthreads();
  if (threadIdx.x == 0) block_counts[blockIdx.x] = s_cnt;
}

// pass 2: exclusive scan of the per-block counts by a single block; total -> counts[nblocks]
__global__ void __launch_bounds__(1024) k_mask_scan(int32_t* counts, int nblocks) {
  __shared__ int s_part[1024];
  const int t = threadIdx.x;
  const int per = (nblocks + 1023) / 1024;
  const int lo = t * per, hi = min(nblocks, lo + per);
  int sum = 0;
  for (int i = lo; i < hi; i++) sum += counts[i];
  s_part[t] = sum;
  __syncthreads();
  for (int o = 1; o < 1024; o <<= 1) {   // Hillis-Steele inclusive scan
    int v = (t >= o) ? s_part[t - o] : 0;
    __syncthreads();
    s_part[t] += v;
    __syncthreads();
  }
  int run = s_part[t] - sum;
  for (int i = lo; i < hi; i++) { int c = counts[i]; counts[i] = run; run += c; }
  if (t == 1023) counts[nblocks] = s_part[1023];
}

// pass 3: scatter pairs, set bits, fill offsets, copy the third column
__global__ void __launch_bounds__(kBuildThreads) k_mask_scatter(const int32_t* items, int64_t n, int V, const int32_t* block_base,
                                                                int nblocks, char* blob, const int32_t* err) {
  if (*err) return;   // a bad table could index out of bounds; the host reports GR_ERR_BAD_TABLE
  const gr_mask_header* h = (const gr_mask_header*)blob;
  uint32_t* l0 = (uint32_t*)(blob + h->off_l0);
  uint32_t* l1 = (uint32_t*)(blob + h->off_l1);
  int32_t* off1 = (int32_t*)(blob + h->off_off1);
  int32_t* pair_off = (int32_t*)(blob + h->off_pair_off);
  int32_t* pair_t2 = (int32_t*)(blob + h->off_pair_t2);
  int32_t* pair_row = (int32_t*)(blob + h->off_pair_row);
  int32_t* t3 = (int32_t*)(blob + h->off_t3);
  const int words = h->words;

  // rows are taken in contiguous runs per thread so that a serial in-thread count gives table order
  __shared__ int s_scan[kBuildThreads];
  const int t = threadIdx.x;
  const int64_t first = (int64_t)blockIdx.x * kRowsPerBlock + (int64_t)t * kRowsPerThread;
  bool nt1[kRowsPerThread], npr[kRowsPerThread];
  int cnt = 0;
  for (int k = 0; k < kRowsPerThread; k++) {
    int64_t i = first + k;
    nt1[k] = npr[k] = false;
    if (i < n) { row_ok_and_flags(items, i, V, &nt1[k], &npr[k]); cnt += npr[k] ? 1 : 0; }
  }
  s_scan[t] = cnt;
  __syncthreads();
  for (int o = 1; o < kBuildThreads; o <<= 1) {
    int v = (t >= o) ? s_scan[t - o] : 0;
    __syncthreads();
    s_scan[t] += v;
    __syncthreads();
  }
  int p = block_base[blockIdx.x] + s_scan[t] - cnt;   // pair index of this thread's first pair start
  const int total_pairs = block_base[nblocks];
  for (int k = 0; k < kRowsPerThread; k++) {
    int64_t i = first + k;
    if (i >= n) break;
    const int32_t a = items[3 * i], b = items[3 * i + 1];
    t3[i] = items[3 * i + 2];
    if (npr[k]) {
      pair_t2[p] = b;
      pair_row[p] = (int32_t)i;
      atomicOr(&l1[(size_t)a * words + (b >> 5)], 1u << (b & 31));
      if (nt1[k]) {
        atomicOr(&l0[a >> 5], 1u << (a & 31));
        const int prev = (i == 0) ? -1 : items[3 * i - 3];
        for (int tok = prev + 1; tok <= a; tok++) { off1[tok] = (int32_t)i; pair_off[tok] = p; }
      }
      p++;
    }
    if (i == n - 1) {
      for (int tok = a + 1; tok <= V; tok++) { off1[tok] = (int32_t)n; pair_off[tok] = total_pairs; }
      pair_row[total_pairs] = (int32_t)n;
      ((gr_mask_header*)blob)->n_pairs = total_pairs;
    }
  }
}

__global__ void k_mask_write_header(char* blob, gr_mask_header h) { *(gr_mask_header*)blob = h; }

}  // namespace

extern "C" size_t gr_item_mask_bytes(int64_t n_items, int32_t depth, int32_t V) {
  if (n_items <= 0 || depth != 3 || V <= 0 || V > 32768) return 0;
  gr_mask_header h;
  gr_mask_layout(n_items, V, &h);
  return (size_t)h.total_bytes;
}

extern "C" size_t gr_item_mask_build_workspace_bytes(int64_t n_items, int32_t depth, int32_t V) {
  if (n_items <= 0 || depth != 3 || V <= 0) return 0;
  int64_t nblocks = (n_items + kRowsPerBlock - 1) / kRowsPerBlock;
  return 256 + gr_align256((size_t)(nblocks + 1) * 4);
}

extern "C" gr_status gr_item_mask_build(const int32_t* items_sorted, int64_t n_items, int32_t depth, int32_t V, void* mask_out,
                                        size_t mask_bytes, void* workspace, size_t workspace_bytes, void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  if (!items_sorted || !mask_out || !workspace || n_items <= 0 || V <= 0) return GR_ERR_INVALID_ARG;
  if (depth != 3 || V > 32768 || n_items >= ((int64_t)1 << 31)) return GR_ERR_UNSUPPORTED;
  if (((uintptr_t)mask_out & 255) || ((uintptr_t)workspace & 255)) return GR_ERR_INVALID_ARG;
  gr_mask_header h;
  gr_mask_layout(n_items, V, &h);
  if (mask_bytes < (size_t)h.total_bytes) return GR_ERR_INVALID_ARG;
  if (workspace_bytes < gr_item_mask_build_workspace_bytes(n_items, depth, V)) return GR_ERR_WORKSPACE_TOO_SMALL;

  char* blob = (char*)mask_out;
  int32_t* err = (int32_t*)workspace;
  int32_t* counts = (int32_t*)((char*)workspace + 256);
  const int nblocks = (int)((n_items + kRowsPerBlock - 1) / kRowsPerBlock);

  hipLaunchKernelGGL(k_mask_write_header, dim3(1), dim3(1), 0, stream, blob, h);
  hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(64), 0, stream, (uint32_t*)err, (size_t)64, 0u);
  // zero the two bitmask levels (they are contiguous in the layout)
  const size_t bit_words = (size_t)(h.off_off1 - h.off_l0) / 4;
  hipLaunchKernelGGL(k_fill_u32, dim3(1024), dim3(256), 0, stream, (uint32_t*)(blob + h.off_l0), bit_words, 0u);
  hipLaunchKernelGGL(k_mask_count, dim3(nblocks), dim3(kBuildThreads), 0, stream, items_sorted, n_items, V, counts, err);
  hipLaunchKernelGGL(k_mask_scan, dim3(1), dim3(1024), 0, stream, counts, nblocks);
  hipLaunchKernelGGL(k_mask_scatter, dim3(nblocks), dim3(kBuildThreads), 0, stream, items_sorted, n_items, V, counts, nblocks, blob, err);
  GR_HIP_TRY(hipGetLastError());
  int32_t host_err = 0;
  GR_HIP_TRY(hipMemcpyAsync(&host_err, err, sizeof(int32_t), hipMemcpyDeviceToHost, stream));
  GR_HIP_TRY(hipStreamSynchronize(stream));
  return host_err ? GR_ERR_BAD_TABLE : GR_OK;
}
