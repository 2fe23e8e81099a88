// gr_beam_attn: shared-prefix beam attention on gfx950 (paper Sections 5.1, 5.2).
//
// Work unit = (request b, KV head h, block of query rows, L segment).  The W*g query rows that share
// KV head h of request b (g = Hq/Hkv) form the N side of a transposed score matrix
//     S^T[kv, q] = K[kv, :] . Q[q, :]          (v_mfma_f32_32x32x16_bf16, A = K tile from LDS, B = Q in registers)
// so that every lane owns ONE query column: the online-softmax max / sum / rescale are per-lane
// scalars and the exponentiated scores leave the accumulators already in the B-operand layout of
//     O^T[d, q] += V^T[d, kv] . P^T[kv, q]     (A = V tile read from LDS with the transposing ds_read_b64_tr_b16).
// Each prompt K/V tile is brought in once per workgroup (direct global -> LDS loads into unpadded, XOR-swizzled
// tiles) and used by all query rows of the block.  The unshared stage (each beam's own u decode tokens) and the merge
// run in the epilogue of segment 0 on the same per-lane state; when the prompt is split into
// segments, partial (max, sum, O) go to the workspace and k_attn_merge combines them.
#include "gr_internal.hpp"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int KT = 64;        // kv tokens per LDS tile
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct AttnCtx {
  int B, W, Hq, Hkv, g, ND, u;
  int M;            // W * g query rows per (b, kv head)
  int MB;           // row blocks per (b, kv head)
  int nsplit;       // L segments per request
  int n_groups;     // B * Hkv * nsplit
  float c;          // sm_scale * log2(e)
  float k_scale, v_scale;   // FP8 prompt cache: value = code * scale (1 for the bf16 cache)
  const uint16_t* q;
  const uint16_t* ks;
  const uint16_t* vs;
  const int32_t* cu;
  const uint16_t* ku;
  const uint16_t* vu;
  uint16_t* out;
  float* lse;
  float* part_o;    // [B, nsplit, W*Hq, D] fp32, unnormalised
  float* part_ml;   // [B, nsplit, W*Hq, 2] (max in log2 domain, sum)
  const int32_t* order;   // [B] requests by decreasing prompt length, or nullptr (requests taken in index order)
  const int32_t* slot;    // [B, W, ND] row of the request's own-token block that holds (beam, token), or nullptr (= w * ND + t)
};

__device__ __forceinline__ float bf16_bits_to_float(uint32_t h) { return __uint_as_float(h << 16); }

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

// n / d and n % d for 0 <= n < 2^22 and a small runtime divisor, through a float reciprocal and one
// correction step (a handful of instructions where the generic 32-bit division takes dozens).
__device__ __forceinline__ void divmod_small(int n, int d, float rcp_d, int* q, int* r) {
  int qq = (int)((float)n * rcp_d);
  int rr = n - qq * d;
  if (rr >= d) { qq++; rr -= d; }
  if (rr < 0) { qq--; rr += d; }
  *q = qq; *r = rr;
}

// Per-tile building blocks.  A tile is KT = 64 prompt tokens; S^T of a tile is [64 kv x 32*NCB q]
// = 2 sub-tiles x NCB column blocks of 32x32 fp32 accumulators.
template <int D, int NCB>
struct AttnTile {
  // Prompt tiles arrive by direct global->LDS loads: a wave-level load writes 1 KiB of consecutive LDS (lane l -> bytes
  // 16 l ..), so tile rows cannot be padded.  Instead the 16-byte pieces of a row are stored permuted (piece p of row r
  // sits in slot p ^ swz(r); the lane that fills slot s fetches piece s ^ swz(r) from memory), chosen so that the
  // operand reads below hit every bank group once:
  //   K (ds_read_b128, 16 lanes = 16 consecutive rows, same piece): swz = r & 15 (256-byte rows) or (r >> 1) & 7 (128-byte rows);
  //   V (ds_read_b64_tr_b16, 32 lanes = 4 consecutive rows x 4 pieces):  swz = 4 (r & 3)  or  4 ((r >> 1) & 1).
  static constexpr int PPRW = D / 8;                                       // 16-byte pieces per row
  static __device__ __forceinline__ int swz_k(int r) { return D == 128 ? (r & 15) : ((r >> 1) & 7); }
  static __device__ __forceinline__ int swz_v(int r) { return D == 128 ? 4 * (r & 3) : 4 * ((r >> 1) & 1); }
  // per-lane element offsets of the operand reads inside a tile (fixed for the whole kernel)
  struct Rd { int k[D / 16]; int v[D / 32]; };
  static __device__ __forceinline__ Rd make_rd(int lane) {
    const int G = lane >> 5, n32 = lane & 31;
    Rd r;
#pragma unroll
    for (int ks = 0; ks < D / 16; ks++) r.k[ks] = n32 * D + ((2 * ks + G) ^ swz_k(n32)) * 8;
    const int vrow = 4 * G + ((lane & 15) >> 2);
#pragma unroll
    for (int db = 0; db < D / 32; db++)
      r.v[db] = vrow * D + ((4 * db + 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1)) ^ swz_v(vrow)) * 8 + 4 * (lane & 1);
    return r;
  }
  static constexpr int KSTR = D + 8;     // padded rows of the Q / output staging and of the own-token mini-tiles (+16 B)
  // V rows: +64 B.  One ds_read_b64_tr_b16 serves 32 lanes per cycle = 4 rows x 2 column halves x 32 bytes; a row
  // stride of 64 B modulo 256 B puts those eight 32-byte groups on eight different bank groups (with +32 B the
  // second half of row r and the first half of row r+1 share banks: a 2-way conflict on every V operand read).
  static constexpr int VSTR = D + 32;    // (own-token mini-tiles only; prompt V tiles are unpadded and swizzled)

  // S^T = K . Q^T from the K tile in LDS (A operand) and Q in registers (B operand)
  static __device__ __forceinline__ void qk(const uint16_t* sk, const bf16x8 (&qop)[NCB][D / 16], f32x16 (&s)[KT / 32][NCB],
                                            const Rd& rdo) {
#pragma unroll
    for (int sub = 0; sub < KT / 32; sub++)
#pragma unroll
      for (int cb = 0; cb < NCB; cb++)
#pragma unroll
        for (int i = 0; i < 16; i++) s[sub][cb][i] = 0.f;
    // operand reads run PF steps ahead of the MFMAs that consume them
    constexpr int N = (KT / 32) * (D / 16), PF = 4;
    bf16x8 a[N];
#pragma unroll
    for (int i = 0; i < PF; i++) a[i] = as_bf16x8(*(const uint4*)(&sk[(i % 2) * 32 * D + rdo.k[i / 2]]));
#pragma unroll
    for (int i = 0; i < N; i++) {
      if (i + PF < N) a[i + PF] = as_bf16x8(*(const uint4*)(&sk[((i + PF) % 2) * 32 * D + rdo.k[(i + PF) / 2]]));
#pragma unroll
      for (int cb = 0; cb < NCB; cb++) s[i % 2][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], qop[cb][i / 2], s[i % 2][cb], 0, 0, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x100, PF, 0);
#pragma unroll
    for (int i = 0; i < N - PF; i++) {
      __builtin_amdgcn_sched_group_barrier(0x008, NCB, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, PF * NCB, 0);
  }

  // O^T += V^T . P^T.  V^T operand: d = 32*db + (lane%32), k slot e <-> token 16*s + 8*(e/4) + 4*G + e%4
  static __device__ __forceinline__ void pv(const uint16_t* sv, const bf16x8 (&pop)[KT / 16][NCB], f32x16 (&o)[D / 32][NCB], const Rd& rdo) {
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    constexpr int N = (KT / 16) * (D / 32), PF = 4;      // operand i: slab i / (D/32), d block i % (D/32)
    auto rd = [&](int i) {
      const uint16_t* p0 = sv + (i / (D / 32)) * 16 * D + rdo.v[i % (D / 32)];
      s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0));
      s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0 + 8 * D));
      s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      return __builtin_bit_cast(bf16x8, both);
    };
    bf16x8 a[N];
#pragma unroll
    for (int i = 0; i < PF; i++) a[i] = rd(i);
#pragma unroll
    for (int i = 0; i < N; i++) {
      if (i + PF < N) a[i + PF] = rd(i + PF);
#pragma unroll
      for (int cb = 0; cb < NCB; cb++)
        o[i % (D / 32)][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], pop[i / (D / 32)][cb], o[i % (D / 32)][cb], 0, 0, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x100, 2 * PF, 1);
#pragma unroll
    for (int i = 0; i < N - PF; i++) {
      __builtin_amdgcn_sched_group_barrier(0x008, NCB, 1);
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 1);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, PF * NCB, 1);
  }

  // Per-lane maximum of a tile's scores for the lane's query column (both halves of the column).
  static __device__ __forceinline__ float colmax(const f32x16 (&s)[KT / 32][NCB]) {
    float mx = -INFINITY;
#pragma unroll
    for (int sub = 0; sub < KT / 32; sub++)
#pragma unroll
      for (int i = 0; i < 16; i += 2) mx = fmaxf(fmaxf(mx, s[sub][0][i]), s[sub][0][i + 1]);
    return fmaxf(mx, __shfl_xor(mx, 32, 64));
  }

  // One steady-state tile with the matrix and vector pipes kept busy together.  The wave issues, in this order,
  // the MFMAs of S(t+1) = K(t+1).Q^T and then those of O += V(t).P(t); between consecutive MFMAs it
  // exponentiates a fixed share of tile t's scores (reference maximum already decided: mc = m_ref * c), so that
  // the 32 quarter-rate exponentials per lane run in the shadow of the 32 MFMAs instead of after them.  P(t) is
  // complete before the second half of the PV MFMAs starts; those are interleaved with the column maximum of
  // S(t+1), which the next tile's decision needs.  Instruction order is pinned chunk by chunk.
  static constexpr int NQK = (KT / 32) * (D / 16), NPV = (KT / 16) * (D / 32), NMF = NQK + NPV;
  static constexpr int EXP_BY = NQK + NPV / 2;            // all 32 exponentials are done after this many MFMAs
  static constexpr int exps_after(int j) {                // exponentials finished once MFMA j's chunk has been issued
    const int t = (32 * (j + 1) + EXP_BY - 1) / EXP_BY;
    return j < 0 ? 0 : (t > 32 ? 32 : t);
  }
  static __device__ __forceinline__ void fused(const uint16_t* sk_next, const uint16_t* sv_cur, const bf16x8 (&qop)[NCB][D / 16],
                                               const f32x16 (&s_cur)[KT / 32][NCB], f32x16 (&s_next)[KT / 32][NCB],
                                               f32x16 (&o)[D / 32][NCB], float mc, float c, float& l_run, float& mx_next, const Rd& rdo) {
    static_assert(NCB == 1, "one column block per wave");
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    auto rdk = [&](int i) { return as_bf16x8(*(const uint4*)(sk_next + (i % 2) * 32 * D + rdo.k[i / 2])); };
    auto rdv = [&](int i) {
      const uint16_t* p0 = sv_cur + (i / (D / 32)) * 16 * D + rdo.v[i % (D / 32)];
      s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0));
      s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0 + 8 * D));
      s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      return __builtin_bit_cast(bf16x8, both);
    };
    constexpr int PF = 4;                                   // operand reads run PF MFMAs ahead
    constexpr int SCAN0 = NMF - NPV / 2, EPC = 32 / (NPV / 2);   // maximum scan: EPC scores per chunk from MFMA SCAN0 on
    bf16x8 a[NMF];
    bf16x8 pop[KT / 16];
    float p[8];
    float rs = 0.f, mx = -INFINITY;
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < PF; i++) a[i] = rdk(i);
#pragma unroll
    for (int j = 0; j < NMF; j++) {
      if (j + PF < NMF) a[j + PF] = (j + PF < NQK) ? rdk(j + PF) : rdv(j + PF - NQK);
      if (j < NQK) {
        s_next[j % 2][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], qop[0][j / 2], j < 2 ? zero : s_next[j % 2][0], 0, 0, 0);
      } else {
        const int i = j - NQK;
        o[i % (D / 32)][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], pop[i / (D / 32)], o[i % (D / 32)][0], 0, 0, 0);
      }
#pragma unroll
      for (int e = exps_after(j - 1); e < exps_after(j); e++) {
        const float v = __builtin_amdgcn_exp2f(fmaf(s_cur[e / 16][0][e % 16], c, -mc));
        rs += v;
        p[e % 8] = v;
        if (e % 8 == 7) {
          bf16x8 pk;
#pragma unroll
          for (int k = 0; k < 8; k += 2) {
            f32x2 two = {p[k], p[k + 1]};
            bf16x2 h = __builtin_convertvector(two, bf16x2);
            pk[k] = h[0];
            pk[k + 1] = h[1];
          }
          pop[e / 8] = pk;
        }
      }
      if (j >= SCAN0) {
#pragma unroll
        for (int e = (j - SCAN0) * EPC; e < (j - SCAN0 + 1) * EPC; e += 2)
          mx = fmaxf(fmaxf(mx, s_next[e / 16][0][e % 16]), s_next[e / 16][0][e % 16 + 1]);
      }
      asm volatile("" : "+v"(rs), "+v"(mx));                 // the running sum and maximum are due here, not at the end of the tile
      __builtin_amdgcn_sched_barrier(0);
    }
    l_run += rs;
    mx_next = fmaxf(mx, __shfl_xor(mx, 32, 64));
  }

  // Online softmax of one tile, one query column per lane (its other half lives in lane^32).
  // The running reference m_ref is only raised when some column of the wave exceeds it by more than
  // kLazy (log2 units): exp2 arguments stay <= kLazy, which fp32 sums and bf16 P hold easily, and the
  // O accumulators need rescaling only on those rare tiles.  Returns (per column block) whether O
  // must be multiplied by alpha[cb].
  static constexpr float kLazy = 8.0f;
  static __device__ __forceinline__ void softmax(f32x16 (&s)[KT / 32][NCB], bf16x8 (&pop)[KT / 16][NCB], float (&m_ref)[NCB],
                                                 float (&l_run)[NCB], float (&alpha)[NCB], bool (&upd)[NCB], float c) {
#pragma unroll
    for (int cb = 0; cb < NCB; cb++) {
      float mx = s[0][cb][0];
#pragma unroll
      for (int sub = 0; sub < KT / 32; sub++)
#pragma unroll
        for (int i = 0; i < 16; i++) mx = fmaxf(mx, s[sub][cb][i]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      upd[cb] = __any(mx * c > m_ref[cb] * c + kLazy);
      const float m_new = upd[cb] ? fmaxf(m_ref[cb], mx) : m_ref[cb];
      alpha[cb] = __builtin_amdgcn_exp2f((m_ref[cb] - m_new) * c);
      const float mc = m_new * c;
      float rs = 0.f;
#pragma unroll
      for (int sub = 0; sub < KT / 32; sub++)
#pragma unroll
        for (int i = 0; i < 16; i++) {
          const float p = __builtin_amdgcn_exp2f(fmaf(s[sub][cb][i], c, -mc));
          s[sub][cb][i] = p;
          rs += p;
        }
      l_run[cb] = l_run[cb] * alpha[cb] + rs;
      m_ref[cb] = m_new;
      // P^T as B operands: slab t = accumulator registers 8*(t%2) .. +7 of sub-tile t/2
#pragma unroll
      for (int t = 0; t < KT / 16; t++) {
        bf16x8 pvv;
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
          f32x2 two = {s[t / 2][cb][8 * (t % 2) + e], s[t / 2][cb][8 * (t % 2) + e + 1]};
          bf16x2 h = __builtin_convertvector(two, bf16x2);
          pvv[e] = h[0];
          pvv[e + 1] = h[1];
        }
        pop[t][cb] = pvv;
      }
    }
  }
};

// CAUSAL = false: the decode step described above.  CAUSAL = true: causal self-attention over the packed prompts
// (the prefill that fills the shared cache, Sections 2.2.1 / 5.1) through the same tiles: request b's query rows are
// its own tokens (row r = token r / g, head r % g of the KV group), a row block only walks the K/V tiles up to its
// last token, scores of keys after a row's token are set to -inf on the tiles that straddle the diagonal, and there
// is no own-token stage and no L split.
// KV8 = true: the prompt K/V are FP8 E4M3 codes with one scale per tensor (value = code * scale).  The tiles are widened
// to bf16 (exactly) on their way into LDS: 8-byte loads into registers one tile ahead, four conversions per 16-byte piece,
// a ds_write into the same swizzled layout the direct loads fill.  The scales never touch the tiles: the K scale goes into
// the exponent scale of the prompt loop, and at the end of the loop the running maximum (x k_scale) and O (x v_scale) are
// put into true units, which is where the bf16 own-token stage and the epilogue work.
template <int D, int NCB, int NWAVES, bool CAUSAL, bool KV8>
__global__ void __launch_bounds__(NWAVES * 64) __attribute__((amdgpu_waves_per_eu(NCB == 1 ? 2 : 1, NCB == 1 ? 2 : 1)))
k_beam_attn(AttnCtx c) {
  using T = AttnTile<D, NCB>;
  constexpr int NT = NWAVES * 64;
  constexpr int MWG = NWAVES * 32 * NCB;
  constexpr int KSTR = T::KSTR, VSTR = T::VSTR;
  constexpr int PPR = D / 8;                     // 16-byte pieces per row
  constexpr int TILE = KT * D;                   // elements of one K or V tile (unpadded, swizzled rows)
  constexpr int NCHUNK = TILE * 2 / 1024;        // 1 KiB chunks (= wave-level loads) per tile
  constexpr int CPW = NCHUNK / NWAVES;           // chunks per wave and tile
  constexpr int RPC = 1024 / (D * 2);            // rows per chunk
  static_assert(NCHUNK % NWAVES == 0, "tile must divide over the waves");
  // double-buffered tiles: K(j) in s_k[j%2], V(j) in s_v[j%2]; then (8-wave workgroups only: they own the CU's LDS
  // anyway) a separate region for the Q hand-over, so that the first tiles can be in flight while Q is staged
  extern __shared__ __attribute__((aligned(1024))) uint16_t smem[];
  uint16_t* s_k = smem;
  uint16_t* s_v = smem + 2 * TILE;
  constexpr bool kQSeparate = NWAVES == 8;
  uint16_t* s_q = kQSeparate ? smem + 4 * TILE : smem;

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, G = lane >> 5, n32 = lane & 31;

  // XCD-aware unit order: workgroups are dealt round-robin to the 8 XCDs, so ids congruent mod 8
  // share an L2.  The MB row blocks that read the same K/V stream get consecutive slots of one XCD.
  // (unsigned arithmetic: these scalar divisions run once per workgroup, but every wave runs them)
  const unsigned id = blockIdx.x;
  const int xcd = (int)(id & 7u);
  const unsigned slot = id >> 3;
  const int group = (int)(slot / (unsigned)c.MB) * 8 + xcd;
  int mbi = (int)(slot % (unsigned)c.MB);
  if (CAUSAL) mbi = c.MB - 1 - mbi;            // the blocks with the most keys to visit start first
  if (group >= c.n_groups) return;
  const unsigned gq = (unsigned)group / (unsigned)c.nsplit;
  const int sp = (int)((unsigned)group - gq * (unsigned)c.nsplit);
  const int bi = (int)(gq / (unsigned)c.Hkv);
  const int kvh = (int)(gq - (unsigned)bi * (unsigned)c.Hkv);
  const int b = c.order ? c.order[bi] : bi;

  const int row0 = c.cu[b];
  const int Lb = c.cu[b + 1] - row0;
  const int Mb = CAUSAL ? Lb * c.g : c.M;                      // query rows of this (request, KV head)
  if (CAUSAL && mbi * (NWAVES * 32 * NCB) >= Mb) return;       // (before any barrier: the whole workgroup leaves)
  int chunk = (int)(((unsigned)Lb + (unsigned)c.nsplit - 1u) / (unsigned)c.nsplit);
  chunk = ((chunk + KT - 1) / KT) * KT;
  const int seg0 = CAUSAL ? 0 : min(Lb, sp * chunk);
  const int seg1 = CAUSAL ? (min((mbi + 1) * (NWAVES * 32 * NCB), Mb) - 1) / c.g + 1 : min(Lb, seg0 + chunk);
  const int ntiles = (seg1 - seg0 + KT - 1) / KT;

  // ---- Q: the workgroup's MWG query rows are fetched with coalesced 16-byte pieces (a row = PPR
  // consecutive lanes) and handed to the lanes that own them through LDS.  A lane reading its own
  // row straight from global memory touches 32 different rows per load instruction, which keeps the
  // address unit busy for microseconds while the CU has nothing else to do.
  static_assert(NCB == 1, "one column block per wave");
  constexpr int QP = MWG * PPR / NT;             // 16-byte pieces of Q per thread
  const float rcp_g = 1.0f / (float)c.g;
  // this request's queries (decode: its W beams; prefill: its own tokens); offsets inside it fit 32 bits
  const uint16_t* q_b = c.q + (CAUSAL ? (size_t)row0 : (size_t)b * c.W) * c.Hq * D;
  uint4 qpiece[QP];
#pragma unroll
  for (int i = 0; i < QP; i++) {
    const int p = tid + i * NT, rl = p / PPR, col = (p % PPR) * 8;
    const int r = mbi * MWG + rl;
    int w, j;
    divmod_small(r, c.g, rcp_g, &w, &j);
    qpiece[i] = make_uint4(0, 0, 0, 0);
    if (r < Mb) qpiece[i] = *(const uint4*)(q_b + (uint32_t)((w * c.Hq + kvh * c.g + j) * D + col));
  }
  int qrow[NCB];       // local query row or -1
  {
    const int r = mbi * MWG + wave * 32 + n32;
    qrow[0] = (r < Mb) ? r : -1;
  }
  // causal mode: the last key a column may see, and the first token of the wave's 32 columns (tiles that end at or
  // before it need no masking).  Columns past the end of the request keep everything (their output is dropped).
  const int tokq = (CAUSAL && qrow[0] >= 0) ? qrow[0] / c.g : 0x7fffffff;
  const int wave_tok0 = CAUSAL ? (mbi * MWG + wave * 32 * NCB) / c.g : 0x7fffffff;

  f32x16 o_acc[D / 32][NCB];
#pragma unroll
  for (int db = 0; db < D / 32; db++)
#pragma unroll
    for (int cb = 0; cb < NCB; cb++)
#pragma unroll
      for (int i = 0; i < 16; i++) o_acc[db][cb][i] = 0.f;
  float m_run[NCB], l_run[NCB];
#pragma unroll
  for (int cb = 0; cb < NCB; cb++) { m_run[cb] = -INFINITY; l_run[cb] = 0.f; }

  // ---- K/V tile staging: global -> LDS directly (no registers, no LDS store instructions).  Wave w fills chunks
  // w, w + NWAVES, ... of a tile: lane l of chunk ch writes LDS bytes 1024 ch + 16 l, i.e. slot l % PPR of row
  // ch * RPC + l / PPR, and therefore fetches piece slot ^ swz(row) of that row.  Rows past the end of the segment
  // (last tile only) re-read the last valid row: finite values that the -inf score mask (K) and zero probabilities
  // (V) make irrelevant.  The loads are issued from inline assembly so that the compiler, which cannot tell the
  // tile buffers apart, does not make every later LDS read wait for them; `tiles_landed` waits for all of this
  // wave's loads, and the barrier that follows publishes every wave's.
  constexpr int EB = KV8 ? 1 : 2;                            // bytes per stored K/V element
  const uint32_t tok_bytes = (uint32_t)c.Hkv * D * EB;      // bytes between consecutive tokens
  const char* kbase = (const char*)c.ks + ((size_t)row0 * c.Hkv + kvh) * D * EB;
  const char* vbase = (const char*)c.vs + ((size_t)row0 * c.Hkv + kvh) * D * EB;
  const float cp = KV8 ? c.c * c.k_scale : c.c;              // exponent scale of the prompt loop
  const typename T::Rd rdo = T::make_rd(lane);
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  int crow[CPW];                                             // this lane's row inside a tile, per chunk
  uint32_t koff[CPW], voff[CPW];                             // and its byte offsets from the tile's first row (full tiles)
#pragma unroll
  for (int i = 0; i < CPW; i++) {
    const int ch = i * NWAVES + wave, row = ch * RPC + lane / PPR, slot = lane % PPR;
    crow[i] = row;
    koff[i] = (uint32_t)row * tok_bytes + (uint32_t)((slot ^ T::swz_k(row)) * 16);
    voff[i] = (uint32_t)row * tok_bytes + (uint32_t)((slot ^ T::swz_v(row)) * 16);
  }
  const uint32_t lds_k = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint16_t*)s_k;
  const uint32_t lds_v = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint16_t*)s_v;
  auto dma = [&](uint32_t lds_addr, const char* gbase, uint32_t off) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(off), "s"(gbase) : "memory", "m0");
  };
  auto tload = [&](bool is_k, int buf, int t) {
    const int tok0 = seg0 + t * KT;                          // wave-uniform
    const char* tile = (is_k ? kbase : vbase) + (size_t)tok0 * tok_bytes;
    const uint32_t lds0 = (is_k ? lds_k : lds_v) + (uint32_t)buf * (TILE * 2);
    const int nvalid = seg1 - tok0;                          // >= 1
    if (nvalid >= KT) {
#pragma unroll
      for (int i = 0; i < CPW; i++) dma(lds0 + (uint32_t)(i * NWAVES + wave_u) * 1024, tile, is_k ? koff[i] : voff[i]);
    } else {
#pragma unroll
      for (int i = 0; i < CPW; i++) {
        const int row = min(crow[i], nvalid - 1), slot = lane % PPR;
        const uint32_t off = (uint32_t)row * tok_bytes + (uint32_t)((slot ^ (is_k ? T::swz_k(crow[i]) : T::swz_v(crow[i]))) * 16);
        dma(lds0 + (uint32_t)(i * NWAVES + wave_u) * 1024, tile, off);
      }
    }
  };
  auto tiles_landed = [&]() { if (!KV8) __builtin_amdgcn_s_waitcnt(0x0F70); };     // vmcnt(0)
  // FP8 tiles: piece p = tid + i * NT of a tile = 8 codes of row p / PPR; registers one tile ahead
  constexpr int P8 = KT * PPR / NT;                          // pieces per thread and tile
  struct Stage8 { uint2 r[P8]; };
  uint32_t off8[P8];                                         // byte offsets of this thread's pieces inside a full tile
#pragma unroll
  for (int i = 0; i < P8; i++) { const int p = tid + i * NT; off8[i] = (uint32_t)(p / PPR) * tok_bytes + (uint32_t)(p % PPR) * 8; }
  auto gload8 = [&](bool is_k, int t) {
    const int tok0 = seg0 + t * KT;
    const char* tile = (is_k ? kbase : vbase) + (size_t)tok0 * tok_bytes;
    const int nvalid = seg1 - tok0;                          // >= 1; rows past the end re-read the last valid row
    Stage8 st;
    if (nvalid >= KT) {
#pragma unroll
      for (int i = 0; i < P8; i++) st.r[i] = *(const uint2*)(tile + off8[i]);
    } else {
#pragma unroll
      for (int i = 0; i < P8; i++) {
        const int p = tid + i * NT, row = min(p / PPR, nvalid - 1), col = p % PPR;
        st.r[i] = *(const uint2*)(tile + (size_t)row * tok_bytes + col * 8);
      }
    }
    return st;
  };
  auto lstore8 = [&](uint16_t* dst, bool is_k, const Stage8& st) {
#pragma unroll
    for (int i = 0; i < P8; i++) {
      const int p = tid + i * NT, row = p / PPR, slot = (p % PPR) ^ (is_k ? T::swz_k(row) : T::swz_v(row));
      const bf16x2 e01 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((int)st.r[i].x, 1.0f, false);
      const bf16x2 e23 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((int)st.r[i].x, 1.0f, true);
      const bf16x2 e45 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((int)st.r[i].y, 1.0f, false);
      const bf16x2 e67 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((int)st.r[i].y, 1.0f, true);
      uint4 v;
      v.x = __builtin_bit_cast(uint32_t, e01); v.y = __builtin_bit_cast(uint32_t, e23);
      v.z = __builtin_bit_cast(uint32_t, e45); v.w = __builtin_bit_cast(uint32_t, e67);
      *(uint4*)(dst + row * D + slot * 8) = v;
    }
  };
  Stage8 k8, v8;

  // ---- geometry of the unshared stage (segment 0 only): every beam's own u decode tokens go through
  // the same MFMA path as the prompt.  The 32 query columns of a wave belong to a handful of beams
  // (32/g of them when g divides 32).  Their K rows (then V rows) form private 32-row mini-tiles,
  // row rho = beam_local * u + token, loaded with coalesced 16-byte pieces into the wave's own slice
  // of the (by then idle) tile memory; S^T = K_u . Q^T is a full 32 x 32 block of which a column
  // keeps only its own beam's u rows (the rest are masked to -inf), and O^T += V_u^T . P^T follows.
  // Compared with per-lane dot products this reads each beam's rows once instead of once per query
  // head and replaces ~1000 VALU operations per lane by 16 MFMAs per wave.  The first mini-tile is
  // fetched into registers while the last prompt tile is still being processed.
  static_assert(NCB == 1, "one column block per wave");
  constexpr int UR = 32;                                 // rows of a mini-tile
  constexpr int UP = UR * PPR / 64;                      // 16-byte pieces per lane and tensor
  const bool own_stage = !CAUSAL && sp == 0 && c.u > 0;
  auto wave_rows = [&](int wv, int* first_beam) {        // rows of wave wv's mini-tiles, and its first beam
    const int r_first = mbi * MWG + wv * 32;
    if (r_first >= Mb) { *first_beam = 0; return 0; }
    const int r_last = min(r_first + 31, Mb - 1);
    *first_beam = r_first / c.g;
    return (r_last / c.g - *first_beam + 1) * c.u;
  };
  int beam0 = 0, npass = 0, R = 0;
  if (own_stage) {
    // the most beams any wave's 32 rows can span (exact when g divides 32, else an upper bound: a surplus
    // pass only sees masked rows)
    const int nb_max = (32 % c.g == 0) ? 32 / c.g : (32 + c.g - 2) / c.g + 1;
    npass = (nb_max * c.u + UR - 1) / UR;
    R = wave_rows(wave, &beam0);
  }
  const int my_lo = (qrow[0] >= 0) ? (qrow[0] / c.g - beam0) * c.u : -1;         // this column's rows [my_lo, my_lo + u)
  uint4 ukp[UP], uvp[UP];
  const float rcp_u = 1.0f / (float)max(c.u, 1);
  auto uload = [&](int pass) {                           // 32 rows x D/8 pieces per tensor; a row = PPR consecutive lanes
    const uint16_t* ku_b = c.ku + (size_t)b * c.W * c.ND * c.Hkv * D;      // this request's own-token caches
    const uint16_t* vu_b = c.vu + (size_t)b * c.W * c.ND * c.Hkv * D;
    const int32_t* slot_b = c.slot ? c.slot + (size_t)b * c.W * c.ND : nullptr;
#pragma unroll
    for (int i = 0; i < UP; i++) {
      const int pi = lane + 64 * i, row = pi / PPR, col = (pi % PPR) * 8;
      const int rho = pass * UR + row;
      ukp[i] = make_uint4(0, 0, 0, 0);
      uvp[i] = make_uint4(0, 0, 0, 0);
      if (rho < R) {
        int bl, tok;
        divmod_small(rho, c.u, rcp_u, &bl, &tok);
        int prow = (beam0 + bl) * c.ND + tok;
        if (slot_b) {                                      // (an entry outside the block falls back to the beam's own row)
          const int sl = slot_b[prow];
          prow = ((unsigned)sl < (unsigned)(c.W * c.ND)) ? sl : prow;
        }
        const uint32_t off = (uint32_t)(prow * (c.Hkv * D) + kvh * D + col);
        ukp[i] = *(const uint4*)(ku_b + off);
        uvp[i] = *(const uint4*)(vu_b + off);
      }
    }
  };

  // first prompt tiles: requested before anything waits on memory (when Q has its own LDS region)
  Stage8 k8b;
  if (KV8) {
    if (ntiles > 0) { k8 = gload8(true, 0); v8 = gload8(false, 0); k8b = gload8(true, min(1, ntiles - 1)); }
  } else if (kQSeparate && ntiles > 0) {
    tload(true, 0, 0); tload(false, 0, 0);
    tload(true, 1, min(1, ntiles - 1));
  }
  // Q as B operands: lane holds query column n32 of the wave's block, d = 16*ks + 8*G + (0..7)
  bf16x8 qop[NCB][D / 16];
  {
#pragma unroll
    for (int i = 0; i < QP; i++) {
      const int p = tid + i * NT, rl = p / PPR, col = (p % PPR) * 8;
      *(uint4*)(&s_q[rl * KSTR + col]) = qpiece[i];
    }
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < D / 16; ks++) qop[0][ks] = as_bf16x8(*(const uint4*)(&s_q[(wave * 32 + n32) * KSTR + ks * 16 + G * 8]));
    if (!kQSeparate) {
      __syncthreads();                               // the tile slots may now be overwritten
      if (!KV8 && ntiles > 0) {
        tload(true, 0, 0); tload(false, 0, 0);
        tload(true, 1, min(1, ntiles - 1));
      }
    }
    if (KV8 && ntiles > 0) {
      lstore8(s_k, true, k8); lstore8(s_v, false, v8); lstore8(s_k + TILE, true, k8b);
      k8 = gload8(true, min(2, ntiles - 1));
      v8 = gload8(false, min(1, ntiles - 1));
    }
  }

  if (ntiles > 0) {
    // Pipeline: iteration t issues S(t+1) = K(t+1).Q^T together with the softmax of S(t), then O += V(t).P(t).
    // K(t+2) and V(t+1) are written to LDS right after the barrier that opens iteration t, so one
    // barrier per tile orders every buffer reuse.  Loads for tiles past the end are clamped to the
    // last tile (harmless re-reads; a duplicate K tile lands in a buffer nobody reads any more).
    const int tl = ntiles - 1;
    tiles_landed();
    __syncthreads();                                   // K(0), V(0), K(1) are in LDS

    auto rescale = [&](const float (&alpha)[NCB], const bool (&upd)[NCB]) {
#pragma unroll
      for (int cb = 0; cb < NCB; cb++)
        if (upd[cb]) {
#pragma unroll
          for (int db = 0; db < D / 32; db++)
#pragma unroll
            for (int i = 0; i < 16; i++) o_acc[db][cb][i] *= alpha[cb];
        }
    };
    // one steady-state iteration: tile t (scores in s_in, column maxima in mx_cur) has a successor whose scores
    // go to s_out.  The reference maximum is settled first (raising it, and rescaling O and the running sum, is a
    // rare wave-uniform branch), so that the tile's MFMAs and exponentials form one straight-line block.
    float mx_cur = -INFINITY;
    auto causal_mask = [&](f32x16 (&s)[KT / 32][NCB], int tok0) {
#pragma unroll
      for (int sub = 0; sub < KT / 32; sub++)
#pragma unroll
        for (int i = 0; i < 16; i++) {
          const int kv = tok0 + sub * 32 + 8 * (i / 4) + 4 * G + (i % 4);
          s[sub][0][i] = (kv > tokq) ? -INFINITY : s[sub][0][i];
        }
    };
    auto step = [&](f32x16 (&s_in)[KT / 32][NCB], f32x16 (&s_out)[KT / 32][NCB], int t) {
      if (CAUSAL && seg0 + t * KT + KT - 1 > wave_tok0) {         // (wave-uniform) this tile reaches past the wave's first token
        causal_mask(s_in, seg0 + t * KT);
        mx_cur = T::colmax(s_in);
      }
      if (__any(mx_cur * cp > m_run[0] * cp + T::kLazy)) {
        const float m_new = fmaxf(m_run[0], mx_cur);
        const float alpha = __builtin_amdgcn_exp2f((m_run[0] - m_new) * cp);
#pragma unroll
        for (int db = 0; db < D / 32; db++)
#pragma unroll
          for (int i = 0; i < 16; i++) o_acc[db][0][i] *= alpha;
        l_run[0] *= alpha;
        m_run[0] = m_new;
      }
      tiles_landed();                                               // this wave's K(t+1) and V(t) loads (issued one step ago)
      __syncthreads();                                              // everyone's; and everyone is done with K(t) and V(t-1)
      if (KV8) {
        lstore8(s_k + (t & 1) * TILE, true, k8);                    // K(t+2) over K(t)
        lstore8(s_v + ((t + 1) & 1) * TILE, false, v8);             // V(t+1) over V(t-1)
        k8 = gload8(true, min(t + 3, tl));
        v8 = gload8(false, min(t + 2, tl));
      } else {
        tload(true, t & 1, min(t + 2, tl));                         // K(t+2) over K(t)
        tload(false, (t + 1) & 1, min(t + 1, tl));                  // V(t+1) over V(t-1)
      }
      T::fused(s_k + ((t + 1) & 1) * TILE, s_v + (t & 1) * TILE, qop, s_in, s_out, o_acc, m_run[0] * cp, cp, l_run[0], mx_cur, rdo);
    };
    // the last tile of the segment: the only one that can be partial, and it has no successor
    auto last = [&](f32x16 (&s_in)[KT / 32][NCB], int t) {
      tiles_landed();
      if (own_stage) uload(0);
      __syncthreads();
      const int tok0 = seg0 + t * KT;
      if (tok0 + KT > seg1) {
#pragma unroll
        for (int sub = 0; sub < KT / 32; sub++)
#pragma unroll
          for (int i = 0; i < 16; i++) {
            const int kv = tok0 + sub * 32 + 8 * (i / 4) + 4 * G + (i % 4);
#pragma unroll
            for (int cb = 0; cb < NCB; cb++) s_in[sub][cb][i] = (kv >= seg1) ? -INFINITY : s_in[sub][cb][i];
          }
      }
      if (CAUSAL) causal_mask(s_in, tok0);
      bf16x8 pop[KT / 16][NCB];
      float alpha[NCB];
      bool upd[NCB];
      T::softmax(s_in, pop, m_run, l_run, alpha, upd, cp);
      rescale(alpha, upd);
      T::pv(s_v + (t & 1) * TILE, pop, o_acc, rdo);
    };

    f32x16 s_a[KT / 32][NCB], s_b[KT / 32][NCB];      // ping-pong score accumulators: no copies
    T::qk(s_k, qop, s_a, rdo);
    if (ntiles > 1) mx_cur = T::colmax(s_a);
    // ntiles - 1 steps, then the last tile.  An odd step is peeled off first so that the loop runs
    // whole ping-pong pairs and the last tile is always in s_a.
    int t = 0;
    if ((ntiles - 1) & 1) {
      step(s_a, s_b, 0);
#pragma unroll
      for (int sub = 0; sub < KT / 32; sub++)
#pragma unroll
        for (int cb = 0; cb < NCB; cb++) s_a[sub][cb] = s_b[sub][cb];
      t = 1;
    }
    for (; t + 1 < ntiles; t += 2) {
      step(s_a, s_b, t);
      step(s_b, s_a, t + 1);
    }
    last(s_a, t);
    if (KV8) {                                         // prompt loop -> true units
      m_run[0] *= c.k_scale;
#pragma unroll
      for (int db = 0; db < D / 32; db++)
#pragma unroll
        for (int i = 0; i < 16; i++) o_acc[db][0][i] *= c.v_scale;
    }
  }

  // ---- unshared stage (segment 0): every beam's own u decode tokens, through the same MFMA path.
  // The 32 query columns of a wave belong to a handful of beams (32/g of them when g divides 32).
  // Their K rows (then V rows) are laid out as private 32-row mini-tiles, row rho = beam_local * u +
  // token, loaded with coalesced 16-byte pieces into the wave's own slice of the (now idle) tile
  // memory; S^T = K_u . Q^T is a full 32 x 32 block of which a column keeps only its own beam's u
  // rows (the rest are masked to -inf), and O^T += V_u^T . P^T follows.  Compared with per-lane dot
  // products this reads each beam's rows once instead of once per query head and replaces ~1000
  // VALU operations per lane by 16 MFMAs per wave.
  if (own_stage) {
    float m = m_run[0], l = l_run[0];
    __syncthreads();                                       // every wave is done with the prompt tiles
    uint16_t* s_uk = smem + wave * UR * KSTR;
    uint16_t* s_uv = smem + NWAVES * UR * KSTR + wave * UR * VSTR;
    if (ntiles == 0) uload(0);
    for (int pass = 0; pass < npass; pass++) {
      if (pass > 0) uload(pass);
#pragma unroll
      for (int i = 0; i < UP; i++) {
        const int pi = lane + 64 * i, row = pi / PPR, col = (pi % PPR) * 8;
        *(uint4*)(&s_uk[row * KSTR + col]) = ukp[i];
        *(uint4*)(&s_uv[row * VSTR + col]) = uvp[i];
      }
      __syncthreads();
      // scores of the 32 rows against the wave's 32 columns
      f32x16 su;
#pragma unroll
      for (int i = 0; i < 16; i++) su[i] = 0.f;
#pragma unroll
      for (int ks = 0; ks < D / 16; ks++) {
        const bf16x8 a = as_bf16x8(*(const uint4*)(&s_uk[n32 * KSTR + ks * 16 + G * 8]));
        su = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qop[0][ks], su, 0, 0, 0);
      }
      // keep the column's own rows; online-softmax update of (m, l, O)
      float mx = -INFINITY;
      bool mine[16];
#pragma unroll
      for (int i = 0; i < 16; i++) {
        const int rho = pass * UR + 8 * (i / 4) + 4 * G + (i % 4);
        mine[i] = my_lo >= 0 && rho >= my_lo && rho < my_lo + c.u;
        if (mine[i]) mx = fmaxf(mx, su[i]);
      }
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m, mx);
      const bool any_key = m_new > -INFINITY;              // false only while the column has seen no key at all
      const float alpha = any_key ? __builtin_amdgcn_exp2f((m - m_new) * c.c) : 1.f;
      float rs = 0.f;
#pragma unroll
      for (int i = 0; i < 16; i++) {
        const float pr = mine[i] ? __builtin_amdgcn_exp2f((su[i] - m_new) * c.c) : 0.f;
        su[i] = pr;
        rs += pr;
      }
      l = l * alpha + rs;
      m = m_new;
#pragma unroll
      for (int db = 0; db < D / 32; db++)
#pragma unroll
        for (int i = 0; i < 16; i++) o_acc[db][0][i] *= alpha;
      bf16x8 pu[UR / 16];
#pragma unroll
      for (int t = 0; t < UR / 16; t++)
#pragma unroll
        for (int e = 0; e < 8; e++) pu[t][e] = (__bf16)su[8 * t + e];
      {
        typedef short s16x8 __attribute__((ext_vector_type(8)));
        const uint16_t* vb = s_uv + (4 * G + ((lane & 15) >> 2)) * VSTR + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
#pragma unroll
        for (int t = 0; t < UR / 16; t++)
#pragma unroll
          for (int db = 0; db < D / 32; db++) {
            const uint16_t* p0 = vb + t * 16 * VSTR + db * 32;
            s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0));
            s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0 + 8 * VSTR));
            s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            o_acc[db][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), pu[t], o_acc[db][0], 0, 0, 0);
          }
      }
      if (pass + 1 < npass) __syncthreads();               // the mini-tiles are rewritten by the next pass
    }
    m_run[0] = m; l_run[0] = l;
  }

  // ---- epilogue: merge is already done in registers; normalise or write this segment's partials
  {
    const int r = qrow[0];
    const float m = m_run[0], l = l_run[0];
    const float l_tot = l + __shfl_xor(l, 32, 64);
    if (c.nsplit == 1) {
      // The wave's 32 rows x D outputs go through its own slice of LDS so that global memory sees whole
      // 256-byte rows (16 lanes x 16 bytes) instead of 8-byte pieces of 32 different rows per store.
      if (!own_stage && ntiles > 0) __syncthreads();       // nobody reads the tile slots any more
      uint16_t* s_o = smem + wave * 32 * KSTR;
      const float inv = (l_tot > 0.f) ? 1.0f / l_tot : 0.f;
#pragma unroll
      for (int db = 0; db < D / 32; db++)
#pragma unroll
        for (int q4 = 0; q4 < 4; q4++) {
          f32x2 a = {o_acc[db][0][4 * q4] * inv, o_acc[db][0][4 * q4 + 1] * inv};
          f32x2 bb = {o_acc[db][0][4 * q4 + 2] * inv, o_acc[db][0][4 * q4 + 3] * inv};
          bf16x2 ha = __builtin_convertvector(a, bf16x2), hb = __builtin_convertvector(bb, bf16x2);
          uint2 st;
          st.x = __builtin_bit_cast(uint32_t, ha);
          st.y = __builtin_bit_cast(uint32_t, hb);
          *(uint2*)(&s_o[n32 * KSTR + db * 32 + 8 * q4 + 4 * G]) = st;
        }
      const float rcp_g2 = 1.0f / (float)c.g;
      uint16_t* out_b = c.out + (CAUSAL ? (size_t)row0 : (size_t)b * c.W) * c.Hq * D;
#pragma unroll
      for (int i = 0; i < 32 * PPR / 64; i++) {
        const int p = lane + 64 * i, rl = p / PPR, col = (p % PPR) * 8;
        const int rr = mbi * MWG + wave * 32 + rl;
        int w, j;
        divmod_small(rr, c.g, rcp_g2, &w, &j);
        const uint4 v = *(const uint4*)(&s_o[rl * KSTR + col]);
        if (rr < Mb) *(uint4*)(out_b + (uint32_t)((w * c.Hq + kvh * c.g + j) * D + col)) = v;
      }
      if (c.lse && G == 0 && r >= 0) {
        int w, j;
        divmod_small(r, c.g, rcp_g2, &w, &j);
        c.lse[((CAUSAL ? (size_t)row0 : (size_t)b * c.W) + w) * c.Hq + kvh * c.g + j] = (l_tot > 0.f) ? (m * c.c + __builtin_amdgcn_logf(l_tot)) * kLn2 : -INFINITY;
      }
    } else {
      // this segment's unnormalised fp32 partial O and (max, sum): staged through LDS like the final
      // output, half of the columns at a time
      if (!own_stage && ntiles > 0) __syncthreads();       // nobody reads the tile slots any more
      float* s_p = (float*)(smem + wave * 32 * KSTR);
      constexpr int CW = D / 2;                            // columns per round: a wave's slice holds 32 rows x CW floats
      constexpr int PSTR = KSTR / 2;                       // floats per staged row (CW + padding)
      const float rcp_g2 = 1.0f / (float)c.g;
      float* part_b = c.part_o + ((size_t)b * c.nsplit + sp) * ((size_t)c.W * c.Hq) * D;
#pragma unroll
      for (int h = 0; h < 2; h++) {
#pragma unroll
        for (int dd = 0; dd < CW / 32; dd++)
#pragma unroll
          for (int q4 = 0; q4 < 4; q4++) {
            const int db = h * (CW / 32) + dd;
            const f32x4 st = {o_acc[db][0][4 * q4], o_acc[db][0][4 * q4 + 1], o_acc[db][0][4 * q4 + 2], o_acc[db][0][4 * q4 + 3]};
            *(f32x4*)(&s_p[n32 * PSTR + dd * 32 + 8 * q4 + 4 * G]) = st;
          }
#pragma unroll
        for (int i = 0; i < CW / 8; i++) {
          const int p = lane + 64 * i, rl = p / (CW / 4), col = (p % (CW / 4)) * 4;
          const int rr = mbi * MWG + wave * 32 + rl;
          int w, j;
          divmod_small(rr, c.g, rcp_g2, &w, &j);
          const f32x4 v = *(const f32x4*)(&s_p[rl * PSTR + col]);
          if (rr < Mb) *(f32x4*)(part_b + (size_t)(w * c.Hq + kvh * c.g + j) * D + h * CW + col) = v;
        }
      }
      if (G == 0 && r >= 0) {
        int w, j;
        divmod_small(r, c.g, rcp_g2, &w, &j);
        const size_t prow = ((size_t)b * c.nsplit + sp) * ((size_t)c.W * c.Hq) + (size_t)w * c.Hq + kvh * c.g + j;
        f32x2 ml = {(l_tot > 0.f) ? m * c.c : -INFINITY, l_tot};
        *(f32x2*)(c.part_ml + prow * 2) = ml;
      }
    }
  }
}

// Merge of the per-segment partials (Section 5.2 merge stage): one wave per output row.
template <int D>
__global__ void __launch_bounds__(256) k_attn_merge(AttnCtx c) {
  const int lane = threadIdx.x & 63;
  const size_t row = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);   // (b, w, hq) flattened
  const size_t rows_per_b = (size_t)c.W * c.Hq;
  if (row >= (size_t)c.B * rows_per_b) return;
  const size_t b = row / rows_per_b, rr = row % rows_per_b;
  float M2 = -INFINITY;
  for (int s = 0; s < c.nsplit; s++) M2 = fmaxf(M2, c.part_ml[((b * c.nsplit + s) * rows_per_b + rr) * 2]);
  float L = 0.f;
  float acc[D / 64];
#pragma unroll
  for (int k = 0; k < D / 64; k++) acc[k] = 0.f;
  for (int s = 0; s < c.nsplit; s++) {
    const size_t prow = (b * c.nsplit + s) * rows_per_b + rr;
    const float m2 = c.part_ml[prow * 2], l = c.part_ml[prow * 2 + 1];
    if (!(l > 0.f)) continue;
    const float sc = __builtin_amdgcn_exp2f(m2 - M2);
    L += l * sc;
#pragma unroll
    for (int k = 0; k < D / 64; k++) acc[k] += c.part_o[prow * D + k * 64 + lane] * sc;
  }
  const float inv = (L > 0.f) ? 1.0f / L : 0.f;
#pragma unroll
  for (int k = 0; k < D / 64; k++) {
    const __bf16 h = (__bf16)(acc[k] * inv);
    c.out[row * D + k * 64 + lane] = __builtin_bit_cast(uint16_t, h);
  }
  if (c.lse && lane == 0) c.lse[row] = (L > 0.f) ? (M2 + __builtin_amdgcn_logf(L)) * kLn2 : -INFINITY;
}

// Requests by decreasing prompt length (ties by index), so that the longest units are dispatched first
// and the tail of a ragged batch is made of short ones.  Rank by counting; B is at most kMaxOrderB.
constexpr int kMaxOrderB = 4096;
__global__ void __launch_bounds__(256) k_attn_order(const int32_t* cu, int B, int32_t* order) {
  __shared__ int s_len[kMaxOrderB];
  for (int i = threadIdx.x; i < B; i += 256) s_len[i] = cu[i + 1] - cu[i];
  __syncthreads();
  for (int i = threadIdx.x; i < B; i += 256) {
    const int li = s_len[i];
    int rank = 0;
    for (int j = 0; j < B; j++) rank += (s_len[j] > li) || (s_len[j] == li && j < i);
    order[rank] = i;
  }
}

// Dynamic LDS of k_beam_attn: K and V tiles, double-buffered (unpadded); the Q hand-over / output staging (padded rows),
// behind the tiles for 256-row workgroups and on top of them for 128-row ones; one padded 32-row K and V mini-tile per
// wave for the own-token stage (on top of everything else, after the prompt loop).
size_t attn_lds_bytes(int d, int mwg) {
  const size_t tiles = (size_t)4 * KT * d * 2;
  const size_t rows = (size_t)mwg * (d + 8) * 2;
  const size_t main_loop = mwg == 256 ? tiles + rows : (tiles > rows ? tiles : rows);
  const size_t own = (size_t)(mwg / 32) * 32 * ((d + 8) + (d + 32)) * 2;
  return main_loop > own ? main_loop : own;
}

// Host-side launch plan, fitted to a measured sweep over (B, L, W) on the MI355X.  8-wave workgroups
// of 256 query rows stage each K/V tile once per 256 rows and win once there are at least 256 of them
// (one per CU); below that, 4-wave workgroups of 128 rows (two fit a CU) fill the chip better than
// splitting the prompt further.  Splitting the prompt into L segments costs fp32 partials through HBM
// plus the merge kernel, so it only pays while it fills idle CUs: segments are added until about one
// workgroup per CU exists (never fewer than four tiles per segment), and not at all once 256 units
// exist without it.
struct AttnPlan { int mwg, nsplit; };
int g_plan_rows = 0, g_plan_segments = 0;                  // gr_diag_attn_plan: 0 = use the rule below
AttnPlan plan_attn(const gr_attn_params* p) {
  const int g = p->Hq / p->Hkv;
  const int64_t M = (int64_t)p->W * g;
  AttnPlan plan;
  if (g_plan_rows) {                                        // a sweep asked for this tiling; keep at least one tile per segment
    const int64_t cap = p->max_L / KT;
    plan.mwg = g_plan_rows;
    plan.nsplit = (int)(g_plan_segments < cap ? g_plan_segments : (cap < 1 ? 1 : cap));
    return plan;
  }
  const int64_t units256 = (int64_t)p->B * p->Hkv * ((M + 255) / 256);
  plan.mwg = (M <= 128 || units256 < 256) ? 128 : 256;     // 256-row workgroups only when they fill the chip by themselves
  const int64_t units = (int64_t)p->B * p->Hkv * ((M + plan.mwg - 1) / plan.mwg);
  plan.nsplit = 1;
  if (units < 256 && p->max_L > 4 * KT) {
    const int64_t want = (256 + units / 2) / units;       // nearest to one workgroup per CU
    const int64_t cap = p->max_L / (4 * KT);              // at least four tiles per segment
    const int64_t n = want < cap ? want : cap;
    plan.nsplit = (int)(n > 16 ? 16 : (n < 1 ? 1 : n));
  }
  return plan;
}

// Ragged batches with more units than CUs are worth ordering by length (measured: 4 % on 128 requests of
// 512..8192 tokens); a uniform batch (total_L == B * max_L) is not touched.
bool attn_wants_order(const gr_attn_params* p, const AttnPlan& plan) {
  const int64_t M = (int64_t)p->W * (p->Hq / p->Hkv);
  const int64_t units = (int64_t)p->B * p->Hkv * ((M + plan.mwg - 1) / plan.mwg) * plan.nsplit;
  return p->B >= 2 && p->B <= kMaxOrderB && p->total_L != (int64_t)p->B * p->max_L && units > 256;
}

}  // namespace

extern "C" gr_status gr_diag_attn_plan(int32_t rows_per_workgroup, int32_t l_segments) {
  if (rows_per_workgroup == 0 && l_segments == 0) { g_plan_rows = g_plan_segments = 0; return GR_OK; }
  if ((rows_per_workgroup != 128 && rows_per_workgroup != 256) || l_segments < 1 || l_segments > 16) return GR_ERR_INVALID_ARG;
  g_plan_rows = rows_per_workgroup; g_plan_segments = l_segments;
  return GR_OK;
}

extern "C" size_t gr_beam_attn_workspace_bytes(const gr_attn_params* p) {
  if (!p || p->B <= 0 || p->W <= 0 || p->Hq <= 0 || p->Hkv <= 0 || p->Hq % p->Hkv) return 0;
  const AttnPlan plan = plan_attn(p);
  size_t need = attn_wants_order(p, plan) ? gr_align256((size_t)p->B * 4) : 0;
  if (plan.nsplit > 1) {
    const size_t rows = (size_t)p->B * plan.nsplit * p->W * p->Hq;
    need += gr_align256(rows * p->d * 4) + gr_align256(rows * 8);
  }
  return need;
}

namespace {
gr_status attn_run(const gr_attn_params* p, const int32_t* slot, bool kv8, float k_scale, float v_scale, void* workspace, size_t workspace_bytes,
                   void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  if (!p) return GR_ERR_INVALID_ARG;
  if (kv8 && (!(k_scale > 0.f) || !(k_scale < INFINITY) || !(v_scale > 0.f) || !(v_scale < INFINITY))) return GR_ERR_INVALID_ARG;
  if (p->B <= 0 || p->W <= 0 || p->Hq <= 0 || p->Hkv <= 0 || p->d <= 0 || p->ND < 0 || p->u < 0 || p->u > p->ND)
    return GR_ERR_INVALID_ARG;
  if (p->max_L < 0 || p->total_L < 0 || p->total_L > (int64_t)p->max_L * p->B) return GR_ERR_INVALID_ARG;
  if (!p->q || !p->cu_seqlens || !p->out) return GR_ERR_INVALID_ARG;
  if (p->total_L > 0 && (!p->k_shared || !p->v_shared)) return GR_ERR_INVALID_ARG;
  if (p->u > 0 && (!p->k_unshared || !p->v_unshared)) return GR_ERR_INVALID_ARG;
  if (p->Hq % p->Hkv) return GR_ERR_INVALID_ARG;
  if ((((uintptr_t)p->q | (uintptr_t)p->k_shared | (uintptr_t)p->v_shared | (uintptr_t)p->k_unshared | (uintptr_t)p->v_unshared |
        (uintptr_t)p->out) & 15) || ((uintptr_t)p->cu_seqlens & 3) || ((uintptr_t)p->lse_out & 3) || ((uintptr_t)slot & 3))
    return GR_ERR_INVALID_ARG;                                                          // every tensor is moved in 16-byte pieces
  if (!(p->sm_scale > 0.f) || !(p->sm_scale < INFINITY)) return GR_ERR_INVALID_ARG;   // (also rejects NaN: the lazy-maximum test assumes a positive scale)
  if (p->d != 64 && p->d != 128) return GR_ERR_UNSUPPORTED;
  if (p->total_L >= ((int64_t)1 << 31)) return GR_ERR_UNSUPPORTED;
  if ((int64_t)p->max_L * p->Hkv * p->d * 2 >= ((int64_t)1 << 32)) return GR_ERR_UNSUPPORTED;   // one request's K (or V) must fit a buffer descriptor
  const int g = p->Hq / p->Hkv;
  if ((int64_t)p->W * g >= ((int64_t)1 << 22)) return GR_ERR_UNSUPPORTED;      // row indices go through divmod_small
  if ((int64_t)p->W * p->Hq * p->d >= ((int64_t)1 << 31) || (int64_t)p->W * p->ND * p->Hkv * p->d >= ((int64_t)1 << 31))
    return GR_ERR_UNSUPPORTED;                                                   // offsets inside one request fit 32 bits

  AttnCtx c;
  c.B = p->B; c.W = p->W; c.Hq = p->Hq; c.Hkv = p->Hkv; c.g = g; c.ND = p->ND; c.u = p->u;
  c.M = p->W * g;
  const AttnPlan plan = plan_attn(p);
  c.MB = (c.M + plan.mwg - 1) / plan.mwg;
  c.nsplit = plan.nsplit;
  c.n_groups = p->B * p->Hkv * c.nsplit;
  c.c = p->sm_scale * kLog2e;
  c.k_scale = kv8 ? k_scale : 1.f; c.v_scale = kv8 ? v_scale : 1.f;
  c.q = (const uint16_t*)p->q; c.ks = (const uint16_t*)p->k_shared; c.vs = (const uint16_t*)p->v_shared;
  c.cu = p->cu_seqlens; c.ku = (const uint16_t*)p->k_unshared; c.vu = (const uint16_t*)p->v_unshared;
  c.out = (uint16_t*)p->out; c.lse = p->lse_out;
  c.part_o = nullptr; c.part_ml = nullptr; c.order = nullptr; c.slot = slot;
  const size_t need = gr_beam_attn_workspace_bytes(p);
  if (need > 0) {
    if (!workspace || ((uintptr_t)workspace & 255)) return GR_ERR_INVALID_ARG;
    if (workspace_bytes < need) return GR_ERR_WORKSPACE_TOO_SMALL;
    char* ws = (char*)workspace;
    if (attn_wants_order(p, plan)) {
      hipLaunchKernelGGL(k_attn_order, dim3(1), dim3(256), 0, stream, p->cu_seqlens, p->B, (int32_t*)ws);
      c.order = (const int32_t*)ws;
      ws += gr_align256((size_t)p->B * 4);
    }
    if (c.nsplit > 1) {
      const size_t rows = (size_t)p->B * c.nsplit * p->W * p->Hq;
      c.part_o = (float*)ws;
      c.part_ml = (float*)(ws + gr_align256(rows * p->d * 4));
    }
  }
  const int64_t groups_padded = ((int64_t)c.n_groups + 7) / 8 * 8;
  const int64_t grid = groups_padded * c.MB;
  if (grid >= ((int64_t)1 << 31)) return GR_ERR_UNSUPPORTED;
  const size_t lds = attn_lds_bytes(p->d, plan.mwg);
#define GR_LAUNCH_ATTN(DD, NCB_, NW_)                                                                                        \
  do {                                                                                                                       \
    if (kv8) {                                                                                                               \
      GR_HIP_TRY(hipFuncSetAttribute((const void*)k_beam_attn<DD, NCB_, NW_, false, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)); \
      hipLaunchKernelGGL((k_beam_attn<DD, NCB_, NW_, false, true>), dim3((unsigned)grid), dim3(NW_ * 64), lds, stream, c);   \
    } else {                                                                                                                 \
      GR_HIP_TRY(hipFuncSetAttribute((const void*)k_beam_attn<DD, NCB_, NW_, false, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)); \
      hipLaunchKernelGGL((k_beam_attn<DD, NCB_, NW_, false, false>), dim3((unsigned)grid), dim3(NW_ * 64), lds, stream, c);  \
    }                                                                                                                        \
  } while (0)
  if (p->d == 128) {
    if (plan.mwg == 256) GR_LAUNCH_ATTN(128, 1, 8); else GR_LAUNCH_ATTN(128, 1, 4);
  } else {
    if (plan.mwg == 256) GR_LAUNCH_ATTN(64, 1, 8); else GR_LAUNCH_ATTN(64, 1, 4);
  }
#undef GR_LAUNCH_ATTN
  if (c.nsplit > 1) {
    const int64_t rows = (int64_t)p->B * p->W * p->Hq;
    const unsigned mgrid = (unsigned)((rows + 3) / 4);
    if (p->d == 128) hipLaunchKernelGGL((k_attn_merge<128>), dim3(mgrid), dim3(256), 0, stream, c);
    else hipLaunchKernelGGL((k_attn_merge<64>), dim3(mgrid), dim3(256), 0, stream, c);
  }
  GR_HIP_TRY(hipGetLastError());
  return GR_OK;
}
}  // namespace

extern "C" gr_status gr_beam_attn(const gr_attn_params* p, void* workspace, size_t workspace_bytes, void* stream) {
  return attn_run(p, nullptr, false, 1.f, 1.f, workspace, workspace_bytes, stream);
}

// The same attention with the own-token caches read through a slot table: nothing is moved between decode steps, the
// table (gr_beam_slot_update) says which row of the request's block holds token t of beam w.
extern "C" gr_status gr_beam_attn_slots(const gr_attn_params* p, const int32_t* slot, void* workspace, size_t workspace_bytes, void* stream) {
  if (!slot) return GR_ERR_INVALID_ARG;
  return attn_run(p, slot, false, 1.f, 1.f, workspace, workspace_bytes, stream);
}

// The same attention over a prompt cache stored as FP8 E4M3 codes with one scale per tensor.
extern "C" gr_status gr_beam_attn_fp8kv(const gr_attn_fp8kv_params* p, void* workspace, size_t workspace_bytes, void* stream) {
  if (!p) return GR_ERR_INVALID_ARG;
  return attn_run(&p->attn, nullptr, true, p->k_scale, p->v_scale, workspace, workspace_bytes, stream);
}

// Causal prompt attention through the same kernel (CAUSAL = true).
extern "C" gr_status gr_prefill_attn(const gr_prefill_params* p, void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  if (!p) return GR_ERR_INVALID_ARG;
  if (p->B <= 0 || p->Hq <= 0 || p->Hkv <= 0 || p->d <= 0 || p->Hq % p->Hkv) return GR_ERR_INVALID_ARG;
  if (p->max_L < 0 || p->total_L < 0 || p->total_L > (int64_t)p->max_L * p->B) return GR_ERR_INVALID_ARG;
  if (!p->cu_seqlens) return GR_ERR_INVALID_ARG;
  if (p->total_L > 0 && (!p->q || !p->k || !p->v || !p->out)) return GR_ERR_INVALID_ARG;
  if ((((uintptr_t)p->q | (uintptr_t)p->k | (uintptr_t)p->v | (uintptr_t)p->out) & 15) || ((uintptr_t)p->cu_seqlens & 3) ||
      ((uintptr_t)p->lse_out & 3))
    return GR_ERR_INVALID_ARG;
  if (!(p->sm_scale > 0.f) || !(p->sm_scale < INFINITY)) return GR_ERR_INVALID_ARG;
  if (p->d != 64 && p->d != 128) return GR_ERR_UNSUPPORTED;
  if (p->total_L >= ((int64_t)1 << 31)) return GR_ERR_UNSUPPORTED;
  if ((int64_t)p->max_L * p->Hkv * p->d * 2 >= ((int64_t)1 << 32)) return GR_ERR_UNSUPPORTED;   // one request's K (or V) must fit a buffer descriptor
  const int g = p->Hq / p->Hkv;
  if ((int64_t)p->max_L * g >= ((int64_t)1 << 22)) return GR_ERR_UNSUPPORTED;                   // row indices go through divmod_small
  if ((int64_t)p->max_L * p->Hq * p->d >= ((int64_t)1 << 31)) return GR_ERR_UNSUPPORTED;        // offsets inside one request fit 32 bits
  if (p->total_L == 0 || p->max_L == 0) return GR_OK;

  AttnCtx c;
  c.B = p->B; c.W = 0; c.Hq = p->Hq; c.Hkv = p->Hkv; c.g = g; c.ND = 0; c.u = 0;
  c.M = p->max_L * g;                                        // the longest request's rows size the grid
  const int mwg = c.M <= 128 ? 128 : 256;
  c.MB = (c.M + mwg - 1) / mwg;
  c.nsplit = 1;
  c.n_groups = p->B * p->Hkv;
  c.c = p->sm_scale * kLog2e;
  c.k_scale = 1.f; c.v_scale = 1.f;
  c.q = (const uint16_t*)p->q; c.ks = (const uint16_t*)p->k; c.vs = (const uint16_t*)p->v;
  c.cu = p->cu_seqlens; c.ku = nullptr; c.vu = nullptr;
  c.out = (uint16_t*)p->out; c.lse = p->lse_out;
  c.part_o = nullptr; c.part_ml = nullptr; c.order = nullptr; c.slot = nullptr;
  const int64_t groups_padded = ((int64_t)c.n_groups + 7) / 8 * 8;
  const int64_t grid = groups_padded * c.MB;
  if (grid >= ((int64_t)1 << 31)) return GR_ERR_UNSUPPORTED;
  const size_t lds = attn_lds_bytes(p->d, mwg);
#define GR_LAUNCH_PREFILL(DD, NW_)                                                                                              \
  do {                                                                                                                         \
    GR_HIP_TRY(hipFuncSetAttribute((const void*)k_beam_attn<DD, 1, NW_, true, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)); \
    hipLaunchKernelGGL((k_beam_attn<DD, 1, NW_, true, false>), dim3((unsigned)grid), dim3(NW_ * 64), lds, stream, c);          \
  } while (0)
  if (p->d == 128) {
    if (mwg == 256) GR_LAUNCH_PREFILL(128, 8); else GR_LAUNCH_PREFILL(128, 4);
  } else {
    if (mwg == 256) GR_LAUNCH_PREFILL(64, 8); else GR_LAUNCH_PREFILL(64, 4);
  }
#undef GR_LAUNCH_PREFILL
  GR_HIP_TRY(hipGetLastError());
  return GR_OK;
}
