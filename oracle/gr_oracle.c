/*
 * CPU oracle for the generative-recommendation decode step (xGR paper).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, obviously-correct statement of
 * what one decode step computes, written the way the paper argues AGAINST doing it on an accelerator:
 *   - attention over a *unified* per-beam KV sequence, the prompt K/V copied for every beam
 *     (paper Section 2.2.2 "redundant memory access", Section 5.1);
 *   - a dense additive item mask built by table membership tests (Section 6.1);
 *   - a full sort of all W*V candidates (Section 6.2, the "partial sorting problem" done in full).
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call it.  It shares no code,
 * header, table or helper with the HIP library.
 *
 * Floating point: attention accumulates in fp64.  The item step follows the canonical rounding
 * documented next to oracle_beam_select() so that a second implementation can reproduce beam
 * indices bit-for-bit.  Compile with -ffp-contract=off.
 *
 * Every function is pinned by tests/test_oracle_*.py against something other than itself
 * (library attention, brute-force enumeration, closed forms, numpy lexsort, invariants).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_ERR_ARG (-1)
#define ORACLE_ERR_MEM (-2)

static float bf16_bits_to_float(uint16_t h) {
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* ------------------------------------------------------------------------------------------------
 * Attention (Section 5.1 cache contents, Section 5.2 what the staged computation must equal).
 *
 * For each requested (request b, beam w, query head hq): build that beam's own contiguous sequence
 *   K_uni = [ prompt K rows of request b ; the beam's u decode-token K rows ]   (same for V)
 * by copying, then textbook softmax attention with KV head hq / (Hq/Hkv):
 *   s_j = sm_scale * <q, K_uni[j]>,  p = softmax(s),  o = sum_j p_j V_uni[j].
 * No causal mask: every key is at or before the query position.
 *
 * q            bf16 bits [B, W, Hq, d]
 * k_sh, v_sh   bf16 bits [total_L, Hkv, d]; request b owns rows cu_seqlens[b] .. cu_seqlens[b+1]-1
 * k_un, v_un   bf16 bits [B, W, ND, Hkv, d]; only the first u token slots are valid
 * triples      int32 [n, 3] = (b, w, hq) rows to compute
 * out          fp64 [n, d];  lse_out fp64 [n] = log sum_j exp(s_j) (natural log), may be NULL
 * ------------------------------------------------------------------------------------------------ */
int oracle_attn_unified(int B, int W, int Hq, int Hkv, int d, int ND, int u, float sm_scale,
                        const uint16_t *q, const uint16_t *k_sh, const uint16_t *v_sh,
                        const int32_t *cu_seqlens, const uint16_t *k_un, const uint16_t *v_un,
                        const int32_t *triples, int64_t n, double *out, double *lse_out) {
    if (B <= 0 || W <= 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || Hq % Hkv != 0 || u < 0 || u > ND)
        return ORACLE_ERR_ARG;
    const int g = Hq / Hkv;
    int status = ORACLE_OK;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t t = 0; t < n; t++) {
        const int b = triples[3 * t], w = triples[3 * t + 1], hq = triples[3 * t + 2];
        if (b < 0 || b >= B || w < 0 || w >= W || hq < 0 || hq >= Hq) { status = ORACLE_ERR_ARG; continue; }
        const int hk = hq / g;
        const int64_t row0 = cu_seqlens[b];
        const int64_t L = (int64_t)cu_seqlens[b + 1] - row0;
        const int64_t n_uni = L + u;
        /* the beam's private, unified copy of its whole KV sequence */
        float *K_uni = (float *)malloc(sizeof(float) * (size_t)n_uni * d);
        float *V_uni = (float *)malloc(sizeof(float) * (size_t)n_uni * d);
        double *s = (double *)malloc(sizeof(double) * (size_t)n_uni);
        if (!K_uni || !V_uni || !s) { status = ORACLE_ERR_MEM; free(K_uni); free(V_uni); free(s); continue; }
        for (int64_t j = 0; j < L; j++)
            for (int c = 0; c < d; c++) {
                K_uni[j * d + c] = bf16_bits_to_float(k_sh[((row0 + j) * Hkv + hk) * d + c]);
                V_uni[j * d + c] = bf16_bits_to_float(v_sh[((row0 + j) * Hkv + hk) * d + c]);
            }
        for (int j = 0; j < u; j++)
            for (int c = 0; c < d; c++) {
                const int64_t src = ((((int64_t)b * W + w) * ND + j) * Hkv + hk) * d + c;
                K_uni[(L + j) * d + c] = bf16_bits_to_float(k_un[src]);
                V_uni[(L + j) * d + c] = bf16_bits_to_float(v_un[src]);
            }
        const uint16_t *qrow = q + (((int64_t)b * W + w) * Hq + hq) * d;
        double smax = -INFINITY;
        for (int64_t j = 0; j < n_uni; j++) {
            double acc = 0.0;
            for (int c = 0; c < d; c++) acc += (double)bf16_bits_to_float(qrow[c]) * (double)K_uni[j * d + c];
            s[j] = (double)sm_scale * acc;
            if (s[j] > smax) smax = s[j];
        }
        double denom = 0.0;
        for (int64_t j = 0; j < n_uni; j++) { s[j] = exp(s[j] - smax); denom += s[j]; }
        for (int c = 0; c < d; c++) {
            double acc = 0.0;
            for (int64_t j = 0; j < n_uni; j++) acc += s[j] * (double)V_uni[j * d + c];
            out[t * d + c] = (n_uni > 0) ? acc / denom : 0.0;
        }
        if (lse_out) lse_out[t] = (n_uni > 0) ? smax + log(denom) : -INFINITY;
        free(K_uni); free(V_uni); free(s);
    }
    return status;
}

/* ------------------------------------------------------------------------------------------------
 * The same unified-cache attention with the prompt K/V given as fp32 values (Section 5.1's shared cache held in
 * a narrower storage format and widened before use: the caller passes the widened values, e.g. FP8 codes times
 * their scale).  Everything else as in oracle_attn_unified: the beam's own decode tokens stay bf16, the beam's
 * sequence is its private copy [prompt ; own tokens], one softmax over all of it, fp64 accumulation.
 *
 * k_sh, v_sh   fp32 [total_L, Hkv, d]
 * ------------------------------------------------------------------------------------------------ */
int oracle_attn_unified_f32kv(int B, int W, int Hq, int Hkv, int d, int ND, int u, float sm_scale,
                              const uint16_t *q, const float *k_sh, const float *v_sh,
                              const int32_t *cu_seqlens, const uint16_t *k_un, const uint16_t *v_un,
                              const int32_t *triples, int64_t n, double *out, double *lse_out) {
    if (B <= 0 || W <= 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || Hq % Hkv != 0 || u < 0 || u > ND)
        return ORACLE_ERR_ARG;
    const int g = Hq / Hkv;
    int status = ORACLE_OK;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t t = 0; t < n; t++) {
        const int b = triples[3 * t], w = triples[3 * t + 1], hq = triples[3 * t + 2];
        if (b < 0 || b >= B || w < 0 || w >= W || hq < 0 || hq >= Hq) { status = ORACLE_ERR_ARG; continue; }
        const int hk = hq / g;
        const int64_t row0 = cu_seqlens[b];
        const int64_t L = (int64_t)cu_seqlens[b + 1] - row0;
        const int64_t n_uni = L + u;
        double *K_uni = (double *)malloc(sizeof(double) * (size_t)(n_uni > 0 ? n_uni : 1) * d);
        double *V_uni = (double *)malloc(sizeof(double) * (size_t)(n_uni > 0 ? n_uni : 1) * d);
        double *s = (double *)malloc(sizeof(double) * (size_t)(n_uni > 0 ? n_uni : 1));
        if (!K_uni || !V_uni || !s) { status = ORACLE_ERR_MEM; free(K_uni); free(V_uni); free(s); continue; }
        for (int64_t j = 0; j < L; j++)
            for (int c = 0; c < d; c++) {
                K_uni[j * d + c] = (double)k_sh[((row0 + j) * Hkv + hk) * d + c];
                V_uni[j * d + c] = (double)v_sh[((row0 + j) * Hkv + hk) * d + c];
            }
        for (int j = 0; j < u; j++)
            for (int c = 0; c < d; c++) {
                const int64_t src = ((((int64_t)b * W + w) * ND + j) * Hkv + hk) * d + c;
                K_uni[(L + j) * d + c] = (double)bf16_bits_to_float(k_un[src]);
                V_uni[(L + j) * d + c] = (double)bf16_bits_to_float(v_un[src]);
            }
        const uint16_t *qrow = q + (((int64_t)b * W + w) * Hq + hq) * d;
        double smax = -INFINITY;
        for (int64_t j = 0; j < n_uni; j++) {
            double acc = 0.0;
            for (int c = 0; c < d; c++) acc += (double)bf16_bits_to_float(qrow[c]) * K_uni[j * d + c];
            s[j] = (double)sm_scale * acc;
            if (s[j] > smax) smax = s[j];
        }
        double denom = 0.0;
        for (int64_t j = 0; j < n_uni; j++) { s[j] = exp(s[j] - smax); denom += s[j]; }
        for (int c = 0; c < d; c++) {
            double acc = 0.0;
            for (int64_t j = 0; j < n_uni; j++) acc += s[j] * V_uni[j * d + c];
            out[t * d + c] = (n_uni > 0) ? acc / denom : 0.0;
        }
        if (lse_out) lse_out[t] = (n_uni > 0) ? smax + log(denom) : -INFINITY;
        free(K_uni); free(V_uni); free(s);
    }
    return status;
}

/* ------------------------------------------------------------------------------------------------
 * Causal self-attention over the prompt (the prefill phase that fills the shared cache: Section 2.2.1
 * "Prefill", Section 5.1; the abstract's claim that prefill and decode go through one staged computation).
 * The textbook definition, one query row at a time: token i of request b, query head hq (KV head hq / g),
 *   s_j = sm_scale * <q_i, k_j>  for the keys j = 0..i of the same request (a token sees itself and what
 *   precedes it), p = softmax(s), o = sum_j p_j v_j.
 *
 * q            bf16 bits [total_L, Hq, d]   (packed: request b owns rows cu_seqlens[b] .. cu_seqlens[b+1]-1)
 * k, v         bf16 bits [total_L, Hkv, d]
 * triples      int32 [n, 3] = (b, i, hq) rows to compute, i relative to the request
 * out          fp64 [n, d];  lse_out fp64 [n] = log sum_{j<=i} exp(s_j), may be NULL
 * ------------------------------------------------------------------------------------------------ */
int oracle_prefill_attn_causal(int B, int Hq, int Hkv, int d, float sm_scale, const uint16_t *q, const uint16_t *k,
                               const uint16_t *v, const int32_t *cu_seqlens, const int32_t *triples, int64_t n,
                               double *out, double *lse_out) {
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || Hq % Hkv != 0) return ORACLE_ERR_ARG;
    const int g = Hq / Hkv;
    int status = ORACLE_OK;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t t = 0; t < n; t++) {
        const int b = triples[3 * t], i = triples[3 * t + 1], hq = triples[3 * t + 2];
        if (b < 0 || b >= B || hq < 0 || hq >= Hq) { status = ORACLE_ERR_ARG; continue; }
        const int64_t row0 = cu_seqlens[b];
        const int64_t L = (int64_t)cu_seqlens[b + 1] - row0;
        if (i < 0 || i >= L) { status = ORACLE_ERR_ARG; continue; }
        const int hk = hq / g;
        const int64_t n_keys = (int64_t)i + 1;
        double *s = (double *)malloc(sizeof(double) * (size_t)n_keys);
        if (!s) { status = ORACLE_ERR_MEM; continue; }
        const uint16_t *qrow = q + ((row0 + i) * Hq + hq) * d;
        double smax = -INFINITY;
        for (int64_t j = 0; j < n_keys; j++) {
            const uint16_t *krow = k + ((row0 + j) * Hkv + hk) * d;
            double acc = 0.0;
            for (int c = 0; c < d; c++) acc += (double)bf16_bits_to_float(qrow[c]) * (double)bf16_bits_to_float(krow[c]);
            s[j] = (double)sm_scale * acc;
            if (s[j] > smax) smax = s[j];
        }
        double denom = 0.0;
        for (int64_t j = 0; j < n_keys; j++) { s[j] = exp(s[j] - smax); denom += s[j]; }
        for (int c = 0; c < d; c++) {
            double acc = 0.0;
            for (int64_t j = 0; j < n_keys; j++) acc += s[j] * (double)bf16_bits_to_float(v[((row0 + j) * Hkv + hk) * d + c]);
            out[t * d + c] = acc / denom;
        }
        if (lse_out) lse_out[t] = smax + log(denom);
        free(s);
    }
    return status;
}

/* ------------------------------------------------------------------------------------------------
 * Item table helpers (Section 6.1: "pre-built valid item vocabulary").
 * The table is int32 [N, depth], rows sorted lexicographically and distinct.  A row is addressed by
 * its packed key  sum_c row[c] * V^(depth-1-c).
 * ------------------------------------------------------------------------------------------------ */
static uint64_t pack_row(const int32_t *row, int depth, int V) {
    uint64_t k = 0;
    for (int c = 0; c < depth; c++) k = k * (uint64_t)V + (uint64_t)row[c];
    return k;
}

/* first table row whose key is >= key */
static int64_t lower_bound_key(const int32_t *items, int64_t N, int depth, int V, uint64_t key) {
    int64_t lo = 0, hi = N;
    while (lo < hi) {
        int64_t mid = lo + (hi - lo) / 2;
        if (pack_row(items + mid * depth, depth, V) < key) lo = mid + 1; else hi = mid;
    }
    return lo;
}

/* Table rows that start with the tokens pre[0..len): [*lo, *hi). */
static void prefix_row_range(const int32_t *items, int64_t N, int depth, int V, const int32_t *pre, int len,
                             int64_t *lo, int64_t *hi) {
    uint64_t base = 0, span = 1;
    for (int c = 0; c < len; c++) base = base * (uint64_t)V + (uint64_t)pre[c];
    for (int c = len; c < depth; c++) { base *= (uint64_t)V; span *= (uint64_t)V; }
    *lo = lower_bound_key(items, N, depth, V, base);
    *hi = lower_bound_key(items, N, depth, V, base + span);
}

/* 0 when the table is sorted, distinct and every token is in [0,V); else 1-based index of the first bad row */
int64_t oracle_check_table(const int32_t *items, int64_t N, int depth, int V) {
    for (int64_t i = 0; i < N; i++) {
        for (int c = 0; c < depth; c++)
            if (items[i * depth + c] < 0 || items[i * depth + c] >= V) return i + 1;
        if (i > 0 && pack_row(items + (i - 1) * depth, depth, V) >= pack_row(items + i * depth, depth, V)) return i + 1;
    }
    return 0;
}

/* Dense additive mask row (Section 6.1): a[v] = 0 if some item starts with prefix + v, else -inf.
 * Decided independently for every v by a binary search over the table. */
int oracle_mask_row(const int32_t *items, int64_t N, int depth, int V, const int32_t *prefix, int len, float *a) {
    if (len < 0 || len >= depth) return ORACLE_ERR_ARG;
    int32_t ext[16];
    if (depth > 16) return ORACLE_ERR_ARG;
    for (int c = 0; c < len; c++) ext[c] = prefix[c];
    for (int v = 0; v < V; v++) {
        int64_t lo, hi;
        ext[len] = v;
        prefix_row_range(items, N, depth, V, ext, len + 1, &lo, &hi);
        a[v] = (hi > lo) ? 0.0f : -INFINITY;
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------------------
 * Beam item step (Sections 2.2.1, 6.1, 6.2): mask, log-softmax over valid tokens, accumulate beam
 * score, keep the best W of the W*V candidates.
 *
 * Canonical arithmetic for a live beam row w (scores_in[w] > -inf) with logits x[v], mask a[v]:
 *   m    = max_v (x[v] + a[v])                         (fp32; exact)
 *   S    = sum_v exp((double)(x[v] + a[v]) - (double)m)  (fp64)
 *   lse  = (float)((double)m + log(S))                 (one rounding to fp32)
 *   bias = scores_in[w] - lse                          (fp32 subtraction)
 *   cand[w*V+v] = bias + x[v]  if a[v] == 0, else -inf  (fp32 addition)
 * Candidates are ordered by (cand descending, flat index w*V+v ascending); output slot j holds the
 * j-th candidate in that order.  Slots past the number of finite candidates are dead:
 * parent = token = -1, score = -inf, prefix all -1, range [0,0), item index -1.
 * A beam whose scores_in is -inf, or that has no valid token, contributes nothing.
 *
 * use_mask == 0: every token is valid (no table needed; ranges and item index come out empty).
 *
 * logits fp32 [B,W,V]; scores_in fp32 [B,W]; prefix_in int32 [B,W,depth] (first `step` entries used)
 * outputs: parent/token int32 [B,W], scores_out fp32 [B,W], prefix_out int32 [B,W,depth],
 *          range_out int32 [B,W,2], item_index_out int32 [B,W] (may be NULL).
 * ------------------------------------------------------------------------------------------------ */
typedef struct { float c; int32_t flat; } cand_t;

static int cand_before(const void *pa, const void *pb) {
    const cand_t *a = (const cand_t *)pa, *b = (const cand_t *)pb;
    if (a->c > b->c) return -1;
    if (a->c < b->c) return 1;
    return (a->flat > b->flat) - (a->flat < b->flat);
}

/* candidates of one request into cand[W*V] (−inf where invalid or dead) */
static int request_candidates(int W, int V, int depth, int step, const int32_t *items, int64_t N, int use_mask,
                              const float *logits, const float *scores_in, const int32_t *prefix_in,
                              cand_t *cand, float *a) {
    for (int w = 0; w < W; w++) {
        const float *x = logits + (int64_t)w * V;
        cand_t *cw = cand + (int64_t)w * V;
        for (int v = 0; v < V; v++) { cw[v].c = -INFINITY; cw[v].flat = w * V + v; }
        if (!(scores_in[w] > -INFINITY)) continue;
        if (use_mask) {
            int rc = oracle_mask_row(items, N, depth, V, prefix_in + (int64_t)w * depth, step, a);
            if (rc) return rc;
        } else {
            for (int v = 0; v < V; v++) a[v] = 0.0f;
        }
        float m = -INFINITY;
        for (int v = 0; v < V; v++) { float xm = x[v] + a[v]; if (xm > m) m = xm; }
        if (!(m > -INFINITY)) continue;
        double S = 0.0;
        for (int v = 0; v < V; v++) S += exp((double)(x[v] + a[v]) - (double)m);
        const float lse = (float)((double)m + log(S));
        const float bias = scores_in[w] - lse;
        for (int v = 0; v < V; v++)
            if (a[v] == 0.0f) cw[v].c = bias + x[v];
    }
    return ORACLE_OK;
}

static void emit_slot(int W, int V, int depth, int step, const int32_t *items, int64_t N, int use_mask,
                      const int32_t *prefix_in, int j, const cand_t *c, int32_t *parent_out, int32_t *token_out,
                      float *scores_out, int32_t *prefix_out, int32_t *range_out, int32_t *item_index_out) {
    (void)W;
    int32_t *po = prefix_out + (int64_t)j * depth;
    for (int k = 0; k < depth; k++) po[k] = -1;
    range_out[2 * j] = 0; range_out[2 * j + 1] = 0;
    if (item_index_out) item_index_out[j] = -1;
    if (!c || !(c->c > -INFINITY)) { parent_out[j] = -1; token_out[j] = -1; scores_out[j] = -INFINITY; return; }
    const int parent = c->flat / V, token = c->flat % V;
    parent_out[j] = parent; token_out[j] = token; scores_out[j] = c->c;
    for (int k = 0; k < step; k++) po[k] = prefix_in[(int64_t)parent * depth + k];
    po[step] = token;
    if (use_mask) {
        int64_t lo, hi;
        prefix_row_range(items, N, depth, V, po, step + 1, &lo, &hi);
        range_out[2 * j] = (int32_t)lo; range_out[2 * j + 1] = (int32_t)hi;
        if (item_index_out && step == depth - 1) item_index_out[j] = (int32_t)lo;
    }
}

int oracle_beam_select(int B, int W, int V, int depth, int step, const int32_t *items, int64_t N, int use_mask,
                       const float *logits, const float *scores_in, const int32_t *prefix_in,
                       int32_t *parent_out, int32_t *token_out, float *scores_out, int32_t *prefix_out,
                       int32_t *range_out, int32_t *item_index_out) {
    if (B <= 0 || W <= 0 || V <= 0 || depth <= 0 || depth > 16 || step < 0 || step >= depth) return ORACLE_ERR_ARG;
    if ((int64_t)W * V > INT32_MAX) return ORACLE_ERR_ARG;
    int status = ORACLE_OK;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; b++) {
        const int64_t n = (int64_t)W * V;
        cand_t *cand = (cand_t *)malloc(sizeof(cand_t) * (size_t)n);
        float *a = (float *)malloc(sizeof(float) * (size_t)V);
        if (!cand || !a) { status = ORACLE_ERR_MEM; free(cand); free(a); continue; }
        const int32_t *pin = prefix_in + (int64_t)b * W * depth;
        int rc = request_candidates(W, V, depth, step, items, N, use_mask, logits + (int64_t)b * n,
                                    scores_in + (int64_t)b * W, pin, cand, a);
        if (rc) { status = rc; free(cand); free(a); continue; }
        qsort(cand, (size_t)n, sizeof(cand_t), cand_before);      /* the full sort */
        for (int j = 0; j < W; j++)
            emit_slot(W, V, depth, step, items, N, use_mask, pin, j, (j < n) ? &cand[j] : NULL,
                      parent_out + (int64_t)b * W, token_out + (int64_t)b * W, scores_out + (int64_t)b * W,
                      prefix_out + (int64_t)b * W * depth, range_out + (int64_t)b * W * 2,
                      item_index_out ? item_index_out + (int64_t)b * W : NULL);
        free(cand); free(a);
    }
    return status;
}

/* ------------------------------------------------------------------------------------------------
 * Second, independent selection: the early-termination walk of Section 6.2.  Each beam's valid
 * candidates are sorted descending on their own; a global min-heap of capacity W holds the best
 * sequences seen so far; beams are visited in order and a beam is abandoned at its first leaf that
 * does not beat the heap's top once the heap is full.  Same outputs as oracle_beam_select;
 * visited_out[b] = number of leaves examined (<= number of valid candidates).
 * ------------------------------------------------------------------------------------------------ */
static int heap_worse(const cand_t *a, const cand_t *b) { return cand_before(a, b) > 0; } /* a ranks after b */

static void heap_sift_down(cand_t *h, int n, int i) {
    for (;;) {
        int l = 2 * i + 1, r = l + 1, worst = i;
        if (l < n && heap_worse(&h[l], &h[worst])) worst = l;
        if (r < n && heap_worse(&h[r], &h[worst])) worst = r;
        if (worst == i) return;
        cand_t t = h[i]; h[i] = h[worst]; h[worst] = t; i = worst;
    }
}

static void heap_sift_up(cand_t *h, int i) {
    while (i > 0) {
        int p = (i - 1) / 2;
        if (!heap_worse(&h[i], &h[p])) return;
        cand_t t = h[i]; h[i] = h[p]; h[p] = t; i = p;
    }
}

int oracle_beam_select_heap(int B, int W, int V, int depth, int step, const int32_t *items, int64_t N, int use_mask,
                            const float *logits, const float *scores_in, const int32_t *prefix_in,
                            int32_t *parent_out, int32_t *token_out, float *scores_out, int32_t *prefix_out,
                            int32_t *range_out, int32_t *item_index_out, int64_t *visited_out) {
    if (B <= 0 || W <= 0 || V <= 0 || depth <= 0 || depth > 16 || step < 0 || step >= depth) return ORACLE_ERR_ARG;
    int status = ORACLE_OK;
    for (int b = 0; b < B; b++) {
        const int64_t n = (int64_t)W * V;
        cand_t *cand = (cand_t *)malloc(sizeof(cand_t) * (size_t)n);
        cand_t *heap = (cand_t *)malloc(sizeof(cand_t) * (size_t)W);
        float *a = (float *)malloc(sizeof(float) * (size_t)V);
        if (!cand || !heap || !a) { free(cand); free(heap); free(a); return ORACLE_ERR_MEM; }
        const int32_t *pin = prefix_in + (int64_t)b * W * depth;
        int rc = request_candidates(W, V, depth, step, items, N, use_mask, logits + (int64_t)b * n,
                                    scores_in + (int64_t)b * W, pin, cand, a);
        if (rc) { free(cand); free(heap); free(a); return rc; }
        int hn = 0;
        int64_t visited = 0;
        for (int w = 0; w < W; w++) {
            cand_t *leaves = cand + (int64_t)w * V;
            qsort(leaves, (size_t)V, sizeof(cand_t), cand_before);      /* this beam's descending list */
            for (int i = 0; i < V; i++) {
                if (!(leaves[i].c > -INFINITY)) break;                  /* end of the valid leaves */
                visited++;
                if (hn < W) { heap[hn] = leaves[i]; heap_sift_up(heap, hn); hn++; continue; }
                if (leaves[i].c > heap[0].c) { heap[0] = leaves[i]; heap_sift_down(heap, hn, 0); }
                else break;                                             /* early termination of this beam */
            }
        }
        qsort(heap, (size_t)hn, sizeof(cand_t), cand_before);
        for (int j = 0; j < W; j++)
            emit_slot(W, V, depth, step, items, N, use_mask, pin, j, (j < hn) ? &heap[j] : NULL,
                      parent_out + (int64_t)b * W, token_out + (int64_t)b * W, scores_out + (int64_t)b * W,
                      prefix_out + (int64_t)b * W * depth, range_out + (int64_t)b * W * 2,
                      item_index_out ? item_index_out + (int64_t)b * W : NULL);
        if (visited_out) visited_out[b] = visited;
        free(cand); free(heap); free(a);
    }
    return status;
}

/* ------------------------------------------------------------------------------------------------
 * In-place reorder of the per-beam decode-token cache by parent index (Section 5.1), stated the
 * plain way: gather into a fresh buffer, then copy back.  new[b, j] = old[b, parent[b, j]];
 * slots with parent < 0 are zero-filled.  kv: bf16 bits [B, W, ND, Hkv, d].
 * ------------------------------------------------------------------------------------------------ */
int oracle_unshared_reorder(int B, int W, int64_t row_elems, const int32_t *parent, uint16_t *kv) {
    uint16_t *tmp = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)W * (size_t)row_elems);
    if (!tmp) return ORACLE_ERR_MEM;
    for (int b = 0; b < B; b++) {
        uint16_t *base = kv + (int64_t)b * W * row_elems;
        for (int j = 0; j < W; j++) {
            int p = parent[(int64_t)b * W + j];
            if (p >= 0 && p < W) memcpy(tmp + (int64_t)j * row_elems, base + (int64_t)p * row_elems, sizeof(uint16_t) * (size_t)row_elems);
            else memset(tmp + (int64_t)j * row_elems, 0, sizeof(uint16_t) * (size_t)row_elems);
        }
        memcpy(base, tmp, sizeof(uint16_t) * (size_t)W * (size_t)row_elems);
    }
    free(tmp);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------------------
 * Second, independent reorder: the in-place procedure Section 5.1 itself describes.  One buffer, no
 * temporary copy of the cache.  Every row j gets a direction index: +1 when its write moves a block
 * upward (the source row parent[j] lies below the target, parent[j] > j), -1 when it moves a block
 * downward (parent[j] < j), 0 when the block stays.  First all upward writes are performed walking
 * down the rows (j increasing), then the remaining writes walking up (j decreasing).
 *
 * The procedure presumes what beam order gives the paper: the live rows come first and their parents
 * are non-decreasing; then no block is overwritten before its last reader has copied it.  Anything
 * else is rejected with ORACLE_ERR_ARG (the buffer is then untouched).  Dead rows (parent < 0), which
 * must follow the live ones, are zero-filled after both sweeps (reading taken here: the paper does
 * not say what a dead slot holds).
 * direction_out: int32 [B, W], may be NULL.
 * ------------------------------------------------------------------------------------------------ */
int oracle_unshared_reorder_two_sweeps(int B, int W, int64_t row_elems, const int32_t *parent, uint16_t *kv,
                                       int32_t *direction_out) {
    if (B <= 0 || W <= 0 || row_elems <= 0) return ORACLE_ERR_ARG;
    for (int b = 0; b < B; b++) {
        const int32_t *p = parent + (int64_t)b * W;
        int n_live = 0;
        while (n_live < W && p[n_live] >= 0) n_live++;
        for (int j = 0; j < W; j++) {
            if (j >= n_live && p[j] >= 0) return ORACLE_ERR_ARG;           /* a live row after a dead one */
            if (j < n_live && p[j] >= W) return ORACLE_ERR_ARG;
            if (j > 0 && j < n_live && p[j] < p[j - 1]) return ORACLE_ERR_ARG; /* parents must not decrease */
        }
    }
    const size_t row_bytes = sizeof(uint16_t) * (size_t)row_elems;
    for (int b = 0; b < B; b++) {
        const int32_t *p = parent + (int64_t)b * W;
        uint16_t *base = kv + (int64_t)b * W * row_elems;
        int n_live = 0;
        while (n_live < W && p[n_live] >= 0) n_live++;
        for (int j = 0; j < W; j++) {
            const int dir = (j >= n_live || p[j] == j) ? 0 : (p[j] > j ? 1 : -1);
            if (direction_out) direction_out[(int64_t)b * W + j] = dir;
        }
        /* upward writes, in downward order */
        for (int j = 0; j < n_live; j++)
            if (p[j] > j) memcpy(base + (int64_t)j * row_elems, base + (int64_t)p[j] * row_elems, row_bytes);
        /* the remaining writes, in upward order */
        for (int j = n_live - 1; j >= 0; j--)
            if (p[j] < j) memcpy(base + (int64_t)j * row_elems, base + (int64_t)p[j] * row_elems, row_bytes);
        for (int j = n_live; j < W; j++) memset(base + (int64_t)j * row_elems, 0, row_bytes);
    }
    return ORACLE_OK;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
