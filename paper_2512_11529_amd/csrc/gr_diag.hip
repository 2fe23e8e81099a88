// Measured machine rates for the benchmark report: a plain streaming read, a loop of back-to-back bf16 MFMAs on
// register operands, and the issue tests (how much vector work, and how many LDS operand reads, ride along with the
// MFMAs on one SIMD).  They give the rates this GPU really reaches under sustained load (power-managed clock, DRAM
// efficiency, shared issue resources), next to which the datasheet figures (8 TB/s, 2.5 PFLOP/s) are quoted.  Not part
// of the decode path.
#include "gr_internal.hpp"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// every workgroup reads one contiguous slice with 16-byte loads, eight in flight per thread
__global__ void __launch_bounds__(256) k_diag_read(const uint4* src, size_t n16_per_block, uint32_t* sink) {
  const uint4* b = src + (size_t)blockIdx.x * n16_per_block;
  uint32_t acc = 0;
  for (size_t i = threadIdx.x; i < n16_per_block; i += 256 * 8) {
    uint4 v[8];
#pragma unroll
    for (int k = 0; k < 8; k++) v[k] = (i + (size_t)k * 256 < n16_per_block) ? b[i + (size_t)k * 256] : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int k = 0; k < 8; k++) acc ^= v[k].x ^ v[k].y ^ v[k].z ^ v[k].w;
  }
  if (acc == 0x9e3779b9u) sink[0] = acc;      // (keeps the loads alive; practically never true)
}

// 8 wavefronts per workgroup, two per SIMD; each keeps kAcc independent accumulator tiles busy
constexpr int kAcc = 4;
__global__ void __launch_bounds__(512) k_diag_mfma(const uint4* operands, int iters, float* sink) {
  const uint4 a4 = operands[threadIdx.x], b4 = operands[512 + threadIdx.x];
  const bf16x8 a = __builtin_bit_cast(bf16x8, a4), b = __builtin_bit_cast(bf16x8, b4);
  f32x16 acc[kAcc];
#pragma unroll
  for (int k = 0; k < kAcc; k++)
#pragma unroll
    for (int i = 0; i < 16; i++) acc[k][i] = 0.f;
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int k = 0; k < kAcc; k++) acc[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[k], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int k = 0; k < kAcc; k++)
#pragma unroll
    for (int i = 0; i < 16; i++) s += acc[k][i];
  if (s == 12345.678f) sink[0] = s;
}

// Issue test: how much vector work hides behind matrix instructions on one SIMD.  Each wavefront iterates
// { one MFMA (four independent accumulator tiles in turn), NV independent fp32 FMAs, NX v_exp_f32 }, in that order.
template <int NV, int NX, bool MFMA>
__global__ void __launch_bounds__(512) k_diag_issue(const uint4* operands, int iters, float* sink) {
  const int lane = threadIdx.x & 63;
  const bf16x8 a = __builtin_bit_cast(bf16x8, operands[threadIdx.x]), b = __builtin_bit_cast(bf16x8, operands[512 + threadIdx.x]);
  f32x16 acc[kAcc];
#pragma unroll
  for (int k = 0; k < kAcc; k++)
#pragma unroll
    for (int i = 0; i < 16; i++) acc[k][i] = 0.f;
  float v[8], x[4];
#pragma unroll
  for (int i = 0; i < 8; i++) v[i] = (float)(lane + i) * 1e-3f;
#pragma unroll
  for (int i = 0; i < 4; i++) x[i] = (float)(lane + i) * 1e-4f;
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int k = 0; k < kAcc; k++) {
      if (MFMA) acc[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[k], 0, 0, 0);
#pragma unroll
      for (int n = 0; n < NV; n++) v[n % 8] = fmaf(v[n % 8], 1.0001f, 1e-6f);
#pragma unroll
      for (int n = 0; n < NX; n++) x[n % 4] = __builtin_amdgcn_exp2f(x[n % 4]) * 1e-3f;
      asm volatile("" : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7]),
                        "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]));
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  float s = 0.f;
#pragma unroll
  for (int k = 0; k < kAcc; k++)
#pragma unroll
    for (int i = 0; i < 16; i++) s += acc[k][i];
#pragma unroll
  for (int i = 0; i < 8; i++) s += v[i];
#pragma unroll
  for (int i = 0; i < 4; i++) s += x[i];
  if (s == 12345.678f) sink[0] = s;
}

// The same loop with the MFMA's A operand read from LDS: every EVERY-th slot (0 = never) takes an operand that a
// conflict-free ds_read_b128 fetched three slots earlier (1 KiB of consecutive LDS per wavefront and read), the other
// slots use registers.  Neither the LDS reads nor the vector work cost anything next to the MFMAs on their own;
// together they do, which is what the attention loop (1.5 operand reads per MFMA) pays.
template <int NV, int NX, int EVERY>
__global__ void __launch_bounds__(512) k_diag_issue_lds(const uint4* operands, int iters, float* sink) {
  __shared__ uint4 tile[4096];                        // 64 rows of 1 KiB
  const int lane = threadIdx.x & 63;
  for (int i = threadIdx.x; i < 4096; i += 512) tile[i] = operands[i & 1023];
  __syncthreads();
  const bf16x8 a = __builtin_bit_cast(bf16x8, operands[threadIdx.x]), b = __builtin_bit_cast(bf16x8, operands[512 + threadIdx.x]);
  f32x16 acc[kAcc];
#pragma unroll
  for (int k = 0; k < kAcc; k++)
#pragma unroll
    for (int i = 0; i < 16; i++) acc[k][i] = 0.f;
  float v[8], x[4];
#pragma unroll
  for (int i = 0; i < 8; i++) v[i] = (float)(lane + i) * 1e-3f;
#pragma unroll
  for (int i = 0; i < 4; i++) x[i] = (float)(lane + i) * 1e-4f;
  uint4 la[3];
#pragma unroll
  for (int i = 0; i < 3; i++) la[i] = tile[64 * i + lane];
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int k = 0; k < 12; k++) {                    // (12 slots per round: the three-deep operand ring and the four accumulators both divide it)
      if (EVERY > 0 && k % EVERY == 0) {
        const int r = (k / EVERY) % 3;
        acc[k % kAcc] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, la[r]), b, acc[k % kAcc], 0, 0, 0);
        la[r] = tile[((k + it) & 63) * 64 + lane];
      } else {
        acc[k % kAcc] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[k % kAcc], 0, 0, 0);
      }
#pragma unroll
      for (int n = 0; n < NV; n++) v[n % 8] = fmaf(v[n % 8], 1.0001f, 1e-6f);
#pragma unroll
      for (int n = 0; n < NX; n++) x[n % 4] = __builtin_amdgcn_exp2f(x[n % 4]) * 1e-3f;
      asm volatile("" : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7]),
                        "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]));
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  float s = 0.f;
#pragma unroll
  for (int k = 0; k < kAcc; k++)
#pragma unroll
    for (int i = 0; i < 16; i++) s += acc[k][i];
#pragma unroll
  for (int i = 0; i < 8; i++) s += v[i];
#pragma unroll
  for (int i = 0; i < 4; i++) s += x[i];
#pragma unroll
  for (int i = 0; i < 3; i++) s += __builtin_bit_cast(float, la[i].x ^ la[i].w);
  if (s == 12345.678f) sink[0] = s;
}

}  // namespace

extern "C" gr_status gr_diag_issue_loop(const void* operands, int32_t workgroups, int32_t iters, int32_t n_fma, int32_t n_exp,
                                        int32_t with_mfma, void* sink, void* stream_) {
  if (!operands || !sink || workgroups <= 0 || iters <= 0 || ((uintptr_t)operands & 15)) return GR_ERR_INVALID_ARG;
  const uint4* ops = (const uint4*)operands;
  float* sk = (float*)sink;
  hipStream_t st = (hipStream_t)stream_;
  const dim3 g((unsigned)workgroups), b(512);
#define GR_ISSUE(NV_, NX_)                                                                                 \
  if (n_fma == NV_ && n_exp == NX_) {                                                                      \
    if (with_mfma) hipLaunchKernelGGL((k_diag_issue<NV_, NX_, true>), g, b, 0, st, ops, iters, sk);        \
    else hipLaunchKernelGGL((k_diag_issue<NV_, NX_, false>), g, b, 0, st, ops, iters, sk);                 \
    GR_HIP_TRY(hipGetLastError());                                                                         \
    return GR_OK;                                                                                          \
  }
  GR_ISSUE(0, 0) GR_ISSUE(2, 0) GR_ISSUE(4, 0) GR_ISSUE(8, 0) GR_ISSUE(12, 0)
  GR_ISSUE(0, 1) GR_ISSUE(2, 1) GR_ISSUE(3, 1) GR_ISSUE(4, 1) GR_ISSUE(4, 2) GR_ISSUE(0, 4)
#undef GR_ISSUE
  return GR_ERR_UNSUPPORTED;
}

extern "C" gr_status gr_diag_issue_loop_lds(const void* operands, int32_t workgroups, int32_t rounds, int32_t n_fma, int32_t n_exp,
                                            int32_t lds_every, void* sink, void* stream_) {
  if (!operands || !sink || workgroups <= 0 || rounds <= 0 || ((uintptr_t)operands & 15)) return GR_ERR_INVALID_ARG;
  const uint4* ops = (const uint4*)operands;
  float* sk = (float*)sink;
  hipStream_t st = (hipStream_t)stream_;
  const dim3 g((unsigned)workgroups), b(512);
#define GR_ISSUE_LDS(NV_, NX_, EV_)                                                                        \
  if (n_fma == NV_ && n_exp == NX_ && lds_every == EV_) {                                                  \
    hipLaunchKernelGGL((k_diag_issue_lds<NV_, NX_, EV_>), g, b, 0, st, ops, rounds, sk);                   \
    GR_HIP_TRY(hipGetLastError());                                                                         \
    return GR_OK;                                                                                          \
  }
  GR_ISSUE_LDS(0, 0, 0) GR_ISSUE_LDS(0, 0, 1) GR_ISSUE_LDS(0, 0, 2)
  GR_ISSUE_LDS(3, 1, 0) GR_ISSUE_LDS(3, 1, 1) GR_ISSUE_LDS(3, 1, 2)
  GR_ISSUE_LDS(5, 0, 0) GR_ISSUE_LDS(5, 0, 1) GR_ISSUE_LDS(0, 2, 0) GR_ISSUE_LDS(0, 2, 1)
#undef GR_ISSUE_LDS
  return GR_ERR_UNSUPPORTED;
}

extern "C" gr_status gr_diag_stream_read(const void* src, size_t bytes, void* sink, void* stream_) {
  if (!src || !sink || bytes < ((size_t)1 << 20) || ((uintptr_t)src & 15)) return GR_ERR_INVALID_ARG;
  const size_t slice = (size_t)32768;                       // bytes per workgroup (one logits row of the headline shape)
  const size_t nblk = bytes / slice;
  if (nblk == 0 || nblk >= ((size_t)1 << 31)) return GR_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(k_diag_read, dim3((unsigned)nblk), dim3(256), 0, (hipStream_t)stream_, (const uint4*)src, slice / 16, (uint32_t*)sink);
  GR_HIP_TRY(hipGetLastError());
  return GR_OK;
}

extern "C" double gr_diag_mfma_flops(int32_t workgroups, int32_t iters) {
  return (double)workgroups * 8.0 * (double)iters * kAcc * 2.0 * 32 * 32 * 16;
}

extern "C" gr_status gr_diag_mfma_loop(const void* operands, int32_t workgroups, int32_t iters, void* sink, void* stream_) {
  if (!operands || !sink || workgroups <= 0 || iters <= 0 || ((uintptr_t)operands & 15)) return GR_ERR_INVALID_ARG;
  hipLaunchKernelGGL(k_diag_mfma, dim3((unsigned)workgroups), dim3(512), 0, (hipStream_t)stream_, (const uint4*)operands, iters, (float*)sink);
  GR_HIP_TRY(hipGetLastError());
  return GR_OK;
}
