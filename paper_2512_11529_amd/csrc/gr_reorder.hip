// gr_beam_reorder: in-place update of the unshared (per-beam) KV cache after a beam step
// (paper Section 5.1): beam j of the new generation continues beam parent[j] of the old one, so
//     cache_new[b, j, 0:u] = cache_old[b, parent[b, j], 0:u]
// inside the one buffer that holds the cache.
//
// The paper orders the row copies (upward moves first, walking down; then the rest, walking up) so
// that no row is overwritten before it is read.  On the GPU the same single-buffer guarantee comes
// from cutting the rows into 128-byte column slices: one workgroup owns one slice of one request,
// gathers that slice of every parent row into registers, passes a barrier, and only then writes the
// slice of every row.  Reads and writes of different workgroups never touch the same bytes, so no
// ordering between workgroups is needed and the permutation may be arbitrary (unsorted parents,
// repeated parents, dead slots).
#include "gr_internal.hpp"

namespace {

constexpr int kReorderThreads = 1024;
constexpr int kSliceBytes = 128;                               // one cache line of each row per workgroup
constexpr int kLanesPerRow = kSliceBytes / 16;                 // 8 lanes x 16 bytes
constexpr int kRowsPerPass = kReorderThreads / kLanesPerRow;   // 128 beams per pass

struct ReorderCtx {
  int W, u;
  uint32_t valid_bytes;     // u * Hkv * d * 2: the live prefix of a beam's row
  size_t row_bytes;         // ND * Hkv * d * 2
  const int32_t* parent;    // [B, W]
  char* k;
  char* v;
};

// NP = passes (rows per thread); W <= NP * kRowsPerPass
template <int NP>
__global__ void __launch_bounds__(kReorderThreads) k_beam_reorder(ReorderCtx c) {
  const int slice = blockIdx.x, b = blockIdx.y;
  char* base = (blockIdx.z == 0 ? c.k : c.v) + (size_t)b * c.W * c.row_bytes;
  const int lane = threadIdx.x % kLanesPerRow, slot = threadIdx.x / kLanesPerRow;
  const uint32_t off = (uint32_t)slice * kSliceBytes + (uint32_t)lane * 16;
  const bool in_row = off < c.valid_bytes;
  uint4 r[NP];
#pragma unroll
  for (int i = 0; i < NP; i++) {
    const int j = slot + i * kRowsPerPass;
    r[i] = make_uint4(0, 0, 0, 0);
    if (in_row && j < c.W) {
      const int p = c.parent[(size_t)b * c.W + j];
      if (p >= 0 && p < c.W) r[i] = *(const uint4*)(base + (size_t)p * c.row_bytes + off);   // dead slots become zeros
    }
  }
  __syncthreads();      // every read of this slice precedes every write of it
#pragma unroll
  for (int i = 0; i < NP; i++) {
    const int j = slot + i * kRowsPerPass;
    if (in_row && j < c.W) *(uint4*)(base + (size_t)j * c.row_bytes + off) = r[i];
  }
}

// The slot table of the alternative that moves no cache bytes: token t of beam j is read from row slot[b][j][t] of the
// request's [W * ND] rows.  After a beam step the new beam j inherits its parent's rows for the tokens both have (t < u)
// and owns row j * ND + t for the tokens still to come; a dead slot (parent outside [0, W)) owns all of its rows.
__global__ void __launch_bounds__(256) k_slot_update(int n, int W, int ND, int u, const int32_t* parent, const int32_t* slot_in, int32_t* slot_out) {
  const int i = blockIdx.x * 256 + threadIdx.x;           // (b, j, t) flattened
  if (i >= n) return;
  const int t = i % ND, bj = i / ND, j = bj % W, b = bj / W;
  int s = j * ND + t;
  if (t < u) {
    const int p = parent[bj];
    if (p >= 0 && p < W) {
      s = p * ND + t;
      if (slot_in) {
        const int sp = slot_in[((size_t)b * W + p) * ND + t];
        s = ((unsigned)sp < (unsigned)(W * ND)) ? sp : s;
      }
    }
  }
  slot_out[i] = s;
}

}  // namespace

extern "C" gr_status gr_beam_slot_update(int32_t B, int32_t W, int32_t ND, int32_t u, const int32_t* parent, const int32_t* slot_in,
                                         int32_t* slot_out, void* stream_) {
  if (B <= 0 || W <= 0 || ND <= 0 || u < 0 || u > ND) return GR_ERR_INVALID_ARG;
  if (!slot_out || slot_in == slot_out || (u > 0 && !parent)) return GR_ERR_INVALID_ARG;
  const int64_t n = (int64_t)B * W * ND;
  if (n >= ((int64_t)1 << 31) || (int64_t)W * ND >= ((int64_t)1 << 31)) return GR_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(k_slot_update, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream_, (int)n, W, ND, u, parent, slot_in,
                     slot_out);
  GR_HIP_TRY(hipGetLastError());
  return GR_OK;
}

extern "C" gr_status gr_beam_reorder(int32_t B, int32_t W, int32_t ND, int32_t Hkv, int32_t d, int32_t u,
                                     const int32_t* parent, void* k_unshared, void* v_unshared, void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  if (B <= 0 || W <= 0 || ND <= 0 || Hkv <= 0 || d <= 0 || u < 0 || u > ND) return GR_ERR_INVALID_ARG;
  if (!parent || !k_unshared || !v_unshared || k_unshared == v_unshared) return GR_ERR_INVALID_ARG;
  if (((uintptr_t)k_unshared & 15) || ((uintptr_t)v_unshared & 15)) return GR_ERR_INVALID_ARG;
  if (((int64_t)Hkv * d * 2) % 16) return GR_ERR_UNSUPPORTED;
  if (W > 16 * kRowsPerPass || B > 65535) return GR_ERR_UNSUPPORTED;
  const int64_t valid = (int64_t)u * Hkv * d * 2;
  if (valid >= ((int64_t)1 << 31)) return GR_ERR_UNSUPPORTED;
  if (u == 0) return GR_OK;
  ReorderCtx c;
  c.W = W; c.u = u;
  c.valid_bytes = (uint32_t)valid;
  c.row_bytes = (size_t)ND * Hkv * d * 2;
  c.parent = parent;
  c.k = (char*)k_unshared; c.v = (char*)v_unshared;
  const dim3 grid((unsigned)((valid + kSliceBytes - 1) / kSliceBytes), (unsigned)B, 2);
  const int np = (W + kRowsPerPass - 1) / kRowsPerPass;
  if (np <= 1) hipLaunchKernelGGL(k_beam_reorder<1>, grid, dim3(kReorderThreads), 0, stream, c);
  else if (np <= 2) hipLaunchKernelGGL(k_beam_reorder<2>, grid, dim3(kReorderThreads), 0, stream, c);
  else if (np <= 4) hipLaunchKernelGGL(k_beam_reorder<4>, grid, dim3(kReorderThreads), 0, stream, c);
  else if (np <= 8) hipLaunchKernelGGL(k_beam_reorder<8>, grid, dim3(kReorderThreads), 0, stream, c);
  else hipLaunchKernelGGL(k_beam_reorder<16>, grid, dim3(kReorderThreads), 0, stream, c);
  GR_HIP_TRY(hipGetLastError());
  return GR_OK;
}
