/*
 * gr.h - C ABI of the MI355X (gfx950) generative-recommendation decode hot path.
 *
 * One decode step of beam-search item generation (xGR paper, arxiv 2512.11529) is
 *   1. attention of all W beam queries of a request over a *separated* KV cache: one shared copy of
 *      the prompt K/V per request plus W short per-beam decode caches (Sections 5.1, 5.2);
 *   2. the beam item step: valid-item mask, log-softmax over valid tokens, cumulative beam score,
 *      and the best W of the W*V candidates (Sections 6.1, 6.2), in fixed caller-owned buffers
 *      (Section 6.3);
 *   3. the move of every surviving beam's own decode cache to its new slot, in place (Section 5.1) - or, moving no
 *      bytes, the update of a slot table that the attention follows (gr_beam_slot_update, gr_beam_attn_slots).
 * Beside the step: the prefill that fills the shared cache (gr_prefill_attn), the step's attention over a shared
 * cache stored in FP8 (gr_beam_attn_fp8kv), an item step for callers that cannot allocate
 * (gr_beam_select_noalloc), and a few diagnostics used by the benchmark (gr_diag_*).
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers unless a comment says "host".  Parameter structs and
 *     scalar arguments are host values read before the call returns.
 *   - The caller owns every buffer, including workspaces and the mask blob.  The library never
 *     allocates, frees or keeps device memory and holds no state between calls (two exceptions, stated
 *     where they are declared: the static scratch array of gr_beam_select_noalloc and the launch-plan
 *     override of gr_diag_attn_plan).
 *   - The attention calls, gr_beam_select and gr_beam_reorder only enqueue kernels on `stream` (a hipStream_t passed as
 *     void*, NULL = default stream); they never synchronise.  gr_item_mask_build is a load-time
 *     call and synchronises `stream` once to report table errors.
 *   - Return value: GR_OK or a negative gr_status.  Nothing is printed, thrown or aborted.
 *     Host-checkable argument errors are reported before anything is enqueued.
 *   - bf16 tensors are raw 16-bit patterns; all tensors are dense, row-major, in the stated shape.
 */
#ifndef GR_H_
#define GR_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t gr_status;
enum {
  GR_OK = 0,
  GR_ERR_INVALID_ARG = -1,        /* NULL pointer, non-positive size, step/u out of range, aliasing rule broken */
  GR_ERR_UNSUPPORTED = -2,        /* shape outside what the kernels implement (see each call) */
  GR_ERR_WORKSPACE_TOO_SMALL = -3,
  GR_ERR_BAD_TABLE = -4,          /* item table unsorted, has duplicates, or a token outside [0, V) */
  GR_ERR_HIP = -5                 /* a HIP runtime call or kernel launch failed */
};

/* Static description of a status code (host pointer, never NULL). */
const char* gr_status_string(gr_status s);

/* ------------------------------------------------------------------------------------------------
 * gr_beam_attn - shared-prefix beam attention (Section 5.1 cache layout, Section 5.2 staging).
 *
 * For every request b, beam w and query head h (KV head h / (Hq/Hkv)) computes softmax attention of
 * q[b,w,h,:] over the L_b prompt tokens of request b (stored ONCE, shared by all W beams) followed
 * by that beam's own u decode tokens:
 *     s_j = sm_scale * <q, k_j>,   out = sum_j softmax(s)_j v_j,   lse = log sum_j exp(s_j).
 * The shared stage streams each prompt K/V tile once per workgroup for many beam queries (bf16
 * MFMA, fp32 accumulation, online softmax); the unshared stage adds each beam's own tokens; the
 * merge combines the (max, sum, output) partials.  No causal mask is applied: every key precedes
 * or is the query position.
 *
 * Supported: d in {64, 128}; Hq % Hkv == 0; 1 <= u <= ND; L_b >= 0 (L_b + u >= 1).  All bf16 tensors must be
 * 16-byte aligned (INVALID_ARG otherwise) and hold finite values.
 * ------------------------------------------------------------------------------------------------ */
typedef struct {
  int32_t B, W, Hq, Hkv, d;   /* requests, beam width, query heads, KV heads, head dim              */
  int32_t ND, u;              /* decode-token capacity per beam (Section 5.1: sized up front) and   */
                              /* number of valid decode tokens this step                            */
  int32_t max_L;              /* host copy of max_b L_b (sizes the launch; no device read-back)     */
  int64_t total_L;            /* host copy of sum_b L_b = cu_seqlens[B]                             */
  float   sm_scale;           /* softmax scale, normally 1/sqrt(d); must be positive and finite     */
  const void*    q;           /* bf16 [B, W, Hq, d]                                                 */
  const void*    k_shared;    /* bf16 [total_L, Hkv, d]; request b = rows cu_seqlens[b]..[b+1]      */
  const void*    v_shared;    /* bf16 [total_L, Hkv, d]                                             */
  const int32_t* cu_seqlens;  /* int32 [B+1], non-decreasing, cu_seqlens[0] = 0                     */
  const void*    k_unshared;  /* bf16 [B, W, ND, Hkv, d]; token slots [0, u) valid                  */
  const void*    v_unshared;  /* bf16 [B, W, ND, Hkv, d]                                            */
  void*          out;         /* bf16 [B, W, Hq, d]                                                 */
  float*         lse_out;     /* fp32 [B, W, Hq] natural-log sum-exp of the scaled scores; or NULL  */
} gr_attn_params;

/* Bytes of workspace gr_beam_attn needs for these shapes (0 is possible).  Host only. */
size_t gr_beam_attn_workspace_bytes(const gr_attn_params* p);

/* Enqueue the attention.  `workspace` (device, 256-byte aligned) holds split-L partials and, for a
 * ragged batch, the order in which requests are dispatched (longest prompt first); contents
 * before and after the call are unspecified.  Errors: INVALID_ARG, UNSUPPORTED,
 * WORKSPACE_TOO_SMALL, HIP. */
gr_status gr_beam_attn(const gr_attn_params* p, void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------------
 * gr_beam_attn_fp8kv - gr_beam_attn over a shared (prompt) cache stored in FP8: the "separated KV cache" of
 * Section 5.1 with its large, read-only half held at one byte per element.  `attn.k_shared` / `attn.v_shared` point
 * to OCP FP8 E4M3 codes, uint8 [total_L, Hkv, d]; the value of an element is code * k_scale (resp. * v_scale),
 * one positive finite scale per tensor.  Everything else (Q, the beams' own decode-token caches, output, workspace,
 * launch rule, errors) is as for gr_beam_attn; the codes are widened to bf16 exactly on their way into LDS and the
 * scales are applied to the scores and to the prompt's share of the output in fp32.
 * ------------------------------------------------------------------------------------------------ */
typedef struct {
  gr_attn_params attn;        /* as for gr_beam_attn, except the element type of k_shared / v_shared */
  float k_scale, v_scale;     /* value = code * scale; must be positive and finite                    */
} gr_attn_fp8kv_params;

/* Workspace: gr_beam_attn_workspace_bytes(&p->attn). */
gr_status gr_beam_attn_fp8kv(const gr_attn_fp8kv_params* p, void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------------
 * gr_prefill_attn - causal self-attention over the packed prompts: the prefill phase that produces the
 * shared cache (Section 2.2.1 "Prefill"; Section 5.1: the shared cache stores the prompt's token-level
 * outputs of the prefill phase; the abstract's single staged computation for prefill and decode).
 *
 * For request b, token i (0 <= i < L_b), query head hq with KV head hq / (Hq/Hkv):
 *     out[i, hq, :] = softmax_j( sm_scale * <q[i, hq], k[j, kvh]> ) . v[j, kvh]   over the keys j = 0..i
 * of the same request.  It runs through the tiles of gr_beam_attn (bf16 MFMA, fp32 accumulation, bf16
 * output): a block of query rows walks the request's K/V tiles up to its own last token and masks
 * the tiles on the diagonal.  No workspace.  Only enqueues on `stream`; no synchronisation.
 *
 * Supported: d in {64, 128}; Hq % Hkv == 0; total_L < 2^31; max_L * Hq/Hkv < 2^22;
 * max_L * Hkv * d * 2 < 2^32; max_L * Hq * d < 2^31.  All bf16 tensors 16-byte aligned.
 * ------------------------------------------------------------------------------------------------ */
typedef struct {
  int32_t B, Hq, Hkv, d;
  int32_t max_L;              /* host copy of max_b L_b (sizes the grid)                             */
  int64_t total_L;            /* host copy of cu_seqlens[B]                                          */
  float   sm_scale;           /* multiplies the scores; must be positive and finite                  */
  const void*    q;           /* bf16 [total_L, Hq, d]  (device), packed like k and v                */
  const void*    k;           /* bf16 [total_L, Hkv, d]                                              */
  const void*    v;           /* bf16 [total_L, Hkv, d]                                              */
  const int32_t* cu_seqlens;  /* int32 [B+1] (device): request b owns rows cu[b] .. cu[b+1]-1        */
  void*          out;         /* bf16 [total_L, Hq, d]                                               */
  float*         lse_out;     /* fp32 [total_L, Hq] natural-log sum-exp of the scaled scores; or NULL */
} gr_prefill_params;

/* Errors: INVALID_ARG, UNSUPPORTED, HIP.  An empty batch (total_L == 0) is GR_OK and launches nothing. */
gr_status gr_prefill_attn(const gr_prefill_params* p, void* stream);

/* ------------------------------------------------------------------------------------------------
 * gr_item_mask_build - valid-item mask, built once at load time (Section 6.1: dense masks are
 * pre-generated during model loading; the last level is kept in sparse form).
 *
 * Input: the table of valid items, int32 [n_items, depth], rows sorted lexicographically and
 * distinct, tokens in [0, V).  Output: one position-independent device blob (offsets, no pointers;
 * may be copied or saved) holding
 *   level 0   bitmask of valid first tokens (V bits);
 *   level 1   dense bitmask of valid second tokens per first token (V x V bits), plus the same
 *             children in sparse CSR form and the table row range of every first token;
 *   level 2   sparse: the third-token column of the table, addressed by row range.
 * The blob is read-only for gr_beam_select and is shared by every step of every request.
 *
 * Supported: depth == 3; 1 <= V <= 32768; 1 <= n_items < 2^31.
 * ------------------------------------------------------------------------------------------------ */
size_t gr_item_mask_bytes(int64_t n_items, int32_t depth, int32_t V);
size_t gr_item_mask_build_workspace_bytes(int64_t n_items, int32_t depth, int32_t V);

/* items_sorted: device int32 [n_items, depth].  mask_out: device, 256-byte aligned, mask_bytes >=
 * gr_item_mask_bytes().  Synchronises `stream`; returns GR_ERR_BAD_TABLE if the on-device check of
 * order / distinctness / token range fails (mask_out is then unspecified). */
gr_status gr_item_mask_build(const int32_t* items_sorted, int64_t n_items, int32_t depth, int32_t V,
                             void* mask_out, size_t mask_bytes, void* workspace, size_t workspace_bytes,
                             void* stream);

/* ------------------------------------------------------------------------------------------------
 * gr_beam_select - beam item step (Sections 6.1-6.3).
 *
 * For each request, for each live beam w (scores_in[w] > -inf) with logits x[v]:
 *     valid(v) = some item starts with (prefix of w, v)                      (mask blob lookup)
 *     m = max over valid x;  S = sum over valid exp(x - m) accumulated in fp64
 *     lse = fp32(m + log S);  bias = scores_in[w] - lse;  cand[w*V+v] = bias + x[v]   (fp32 ops)
 * and the W best candidates by (cand descending, flat index w*V+v ascending) are written, best
 * first.  Selection stops reading as soon as the W survivors are fixed (threshold filtering
 * instead of a sort of all W*V candidates - the early-termination idea of Section 6.2).
 * Slots past the number of finite candidates are dead: parent = token = -1, score = -inf,
 * prefix = -1, range = [0,0), item index = -1.
 *
 * Prefix state carried between steps (Section 6.3: fixed-size structures, overwritten in place by
 * the caller swapping in/out buffers):
 *   prefix  int32 [B, W, depth]  tokens chosen so far (entries >= step+1 are -1 on output)
 *   range   int32 [B, W, 2]      table row range [lo, hi) of the prefix
 * Step 0 ignores prefix_in/range_in.  Step 1 reads prefix_in[...,0]; step 2 reads range_in.
 * Behaviour is undefined if logits or scores contain NaN, or if a live beam's prefix/range is not
 * one this mask produced.
 *
 * mask == NULL: unconstrained (every token valid); range_out = [0,0), item_index_out = -1.
 * Supported: depth == 3; 1 <= W <= 2048; 1 <= V <= 32768; W*V < 2^31.
 * ------------------------------------------------------------------------------------------------ */
enum {
  GR_SELECT_FORCE_DENSE = 1     /* stream every live row in full even when a sparse gather would be cheaper */
};

typedef struct {
  int32_t B, W, V, depth, step;   /* 0 <= step < depth                                              */
  int32_t flags;                  /* GR_SELECT_* bits                                               */
  const void*    mask;            /* blob from gr_item_mask_build (built for the same V, depth)     */
  const float*   logits;          /* fp32 [B, W, V]                                                 */
  const float*   scores_in;       /* fp32 [B, W]; -inf = dead beam                                  */
  const int32_t* prefix_in;       /* int32 [B, W, depth]                                            */
  const int32_t* range_in;        /* int32 [B, W, 2]                                                */
  int32_t*       parent_out;      /* int32 [B, W] index of the beam each survivor extends           */
  int32_t*       token_out;       /* int32 [B, W] token appended                                    */
  float*         scores_out;      /* fp32 [B, W] cumulative log-probability, non-increasing         */
  int32_t*       prefix_out;      /* int32 [B, W, depth]; must not alias prefix_in                  */
  int32_t*       range_out;       /* int32 [B, W, 2];     must not alias range_in                   */
  int32_t*       item_index_out;  /* int32 [B, W] table row of the finished item when step ==       */
                                  /* depth-1 (else -1); may be NULL                                 */
} gr_select_params;

size_t gr_beam_select_workspace_bytes(int32_t B, int32_t W, int32_t V, int32_t depth);

/* Enqueue the item step.  `workspace`: device, 256-byte aligned, contents unspecified before and
 * after.  Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE_TOO_SMALL, HIP. */
gr_status gr_beam_select(const gr_select_params* p, void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------------
 * gr_beam_select_noalloc - gr_beam_select for callers that cannot allocate device memory or carry a
 * workspace around: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 *
 * Same parameters, same results and same errors as gr_beam_select; the workspace is a static device array
 * inside the library (gr_beam_select_noalloc_max_workspace_bytes() bytes, 16 MiB: on every GPU the library
 * runs on until the process ends).  A shape whose gr_beam_select_workspace_bytes() exceeds that limit is
 * rejected with GR_ERR_WORKSPACE_TOO_SMALL before anything is enqueued (at V = 8192 the limit is about 16 000
 * beam rows, B * W).  The call allocates nothing and frees nothing; the first call on a device looks up the
 * array's address on that device (no synchronisation).  All calls on one GPU share the array: calls that
 * overlap in time on one GPU (different streams, different host threads) race and give undefined results -
 * order them, or use gr_beam_select with separate workspaces.
 * ------------------------------------------------------------------------------------------------ */
size_t    gr_beam_select_noalloc_max_workspace_bytes(void);
gr_status gr_beam_select_noalloc(const gr_select_params* p, void* stream);

/* ------------------------------------------------------------------------------------------------
 * gr_beam_reorder - in-place update of the unshared cache between two decode steps (Section 5.1).
 *
 * After gr_beam_select, slot j of the new beam generation continues old beam parent[b, j].  The
 * per-beam decode cache follows it inside the single buffer that holds it (no second copy):
 *     cache[b, j, t, :, :] <- cache[b, parent[b, j], t, :, :]     for token slots t in [0, u)
 * for both K and V.  Slots with parent < 0 (dead beams) are zero-filled; token slots >= u are left
 * untouched (the caller writes slot u next).  The paper orders row moves by direction so that no
 * block is overwritten before it is read; this call gives the same guarantee for any parent
 * array (unsorted, repeated parents) by gathering before a barrier and writing after it.
 *
 * parent: device int32 [B, W] (gr_beam_select's parent_out).  k_unshared, v_unshared: device bf16
 * [B, W, ND, Hkv, d], 16-byte aligned, distinct buffers, modified in place.  Only enqueues on
 * `stream`.  Supported: W <= 2048; B <= 65535; Hkv*d a multiple of 8.  Errors: INVALID_ARG,
 * UNSUPPORTED, HIP.
 * ------------------------------------------------------------------------------------------------ */
gr_status gr_beam_reorder(int32_t B, int32_t W, int32_t ND, int32_t Hkv, int32_t d, int32_t u,
                          const int32_t* parent, void* k_unshared, void* v_unshared, void* stream);

/* ------------------------------------------------------------------------------------------------
 * gr_beam_slot_update / gr_beam_attn_slots - the same hand-over of the unshared cache between decode steps
 * (Section 5.1) without moving any cache bytes.
 *
 * The paper moves each surviving beam's rows to its new place.  Here the rows stay where they were written and a
 * slot table follows the beams instead: token t of beam w of request b is read from row slot[b, w, t] of that
 * request's [W * ND] rows of k_unshared / v_unshared (the same [B, W, ND, Hkv, d] buffers, seen as B blocks of
 * W * ND rows).  A row is written once - the caller writes the K/V of beam j's token t to row j * ND + t, as for
 * gr_beam_attn - and never overwritten afterwards, because position t only ever receives tokens of step t.
 *
 * gr_beam_slot_update: slot_out[b, j, t] = slot_in[b, parent[b, j], t] for t < u (the tokens the new beam shares
 *   with its parent); = j * ND + t for t >= u (its own rows, where the next tokens go) and for every t of a dead
 *   slot (parent outside [0, W)).  slot_in == NULL means the identity table (before the first beam step).  parent:
 *   device int32 [B, W]; slot_in, slot_out: device int32 [B, W, ND], distinct.  u = tokens per beam before the
 *   step that produced `parent`, 0 <= u <= ND.
 * gr_beam_attn_slots: gr_beam_attn with `slot` (device int32 [B, W, ND], required) applied to every read of
 *   k_unshared / v_unshared; an entry outside [0, W * ND) is read as the identity entry instead of being followed.
 *   Same parameters, workspace, launch rule and results as gr_beam_attn on a cache reordered by gr_beam_reorder
 *   (bit for bit for live beams).
 * Both only enqueue on `stream`.  Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE_TOO_SMALL, HIP.
 * ------------------------------------------------------------------------------------------------ */
gr_status gr_beam_slot_update(int32_t B, int32_t W, int32_t ND, int32_t u, const int32_t* parent, const int32_t* slot_in,
                              int32_t* slot_out, void* stream);
gr_status gr_beam_attn_slots(const gr_attn_params* p, const int32_t* slot, void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------------
 * Diagnostics: the rates this GPU really sustains, reported by the benchmark next to the datasheet peaks
 * (the evaluation quotes achieved rates against the hardware's capability; Section 9.4).  Not part of the
 * decode path.  Both only enqueue on `stream`.
 *
 * gr_diag_stream_read: reads `bytes` (>= 1 MiB, 16-byte aligned device memory; whole 32 KiB slices are read)
 *   with 16-byte loads and discards them; `sink` is 4 writable device bytes.
 * gr_diag_mfma_loop: `workgroups` x 8 wavefronts each issue `iters` x 4 back-to-back bf16 32x32x16 MFMAs on the
 *   operands found at `operands` (16 KiB of device memory: 2 x 512 x 16 bytes of bf16); `sink` is 4 writable
 *   device bytes.  gr_diag_mfma_flops gives the floating-point operations of such a launch (host only).
 * gr_diag_attn_plan: host only, process-wide.  Makes every later gr_beam_attn / gr_beam_attn_workspace_bytes use
 *   workgroups of `rows_per_workgroup` (128 or 256) query rows and `l_segments` (1..16, lowered to the number of
 *   K/V tiles in the longest prompt) prompt segments instead of the built-in launch rule; (0, 0) restores the rule.
 *   For sweeps that refit the rule; not thread-safe against concurrent gr_beam_attn calls.
 * gr_diag_issue_loop: the issue test behind the attention kernel's roofline discussion.  `workgroups` x 8 wavefronts
 *   (256 workgroups = two wavefronts per SIMD, 512 = four) each run `iters` x 4 slots of { one bf16 32x32x16 MFMA if
 *   `with_mfma`, `n_fma` independent fp32 FMAs, `n_exp` v_exp_f32 }.  Built combinations (n_fma, n_exp): (0,0) (2,0)
 *   (4,0) (8,0) (12,0) (0,1) (2,1) (3,1) (4,1) (4,2) (0,4); others return UNSUPPORTED.  Operands and sink as for
 *   gr_diag_mfma_loop.
 * gr_diag_issue_loop_lds: the same test with the MFMA's first operand coming from LDS, as the attention loop's K and V
 *   operands do: `rounds` x 12 slots per wavefront; every `lds_every`-th slot (0 = never, 1, 2) uses an operand that a
 *   conflict-free ds_read_b128 fetched three slots earlier.  Built (n_fma, n_exp, lds_every): (0,0,*) (3,1,*) (5,0,0)
 *   (5,0,1) (0,2,0) (0,2,1).  Uses 64 KiB of LDS per workgroup.
 * Errors: INVALID_ARG, UNSUPPORTED, HIP.
 * ------------------------------------------------------------------------------------------------ */
gr_status gr_diag_issue_loop(const void* operands, int32_t workgroups, int32_t iters, int32_t n_fma, int32_t n_exp,
                             int32_t with_mfma, void* sink, void* stream);
gr_status gr_diag_issue_loop_lds(const void* operands, int32_t workgroups, int32_t rounds, int32_t n_fma, int32_t n_exp,
                                 int32_t lds_every, void* sink, void* stream);
gr_status gr_diag_attn_plan(int32_t rows_per_workgroup, int32_t l_segments);
gr_status gr_diag_stream_read(const void* src, size_t bytes, void* sink, void* stream);
gr_status gr_diag_mfma_loop(const void* operands, int32_t workgroups, int32_t iters, void* sink, void* stream);
double    gr_diag_mfma_flops(int32_t workgroups, int32_t iters);

#ifdef __cplusplus
}
#endif
#endif /* GR_H_ */
