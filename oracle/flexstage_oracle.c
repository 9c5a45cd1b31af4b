/*
 * flexstage CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * stage-forward and KV-repartition paths compute.  Only the test-suite, the
 * smoke check and the benchmark's cpu_baseline leg may build, load or call it;
 * the GPU library never does, and the two share no source.
 *
 * What is stated here, and where the paper asks for it:
 *   - one pipeline stage = a contiguous range of decoder layers run over a
 *     dynamic batch (Section 3.2, Table 2 "Compute"; Section 5, the partition
 *     constraints of Eq. 2: stages are a disjoint cover of the operator graph,
 *     so running stage [a,k) then [k,b) is the same function as [a,b));
 *   - the KV cache of every layer follows the layer to its new owner when the
 *     stage boundaries move, carrying only valid tokens (Section 6.3, Eq. 10:
 *     KV (x) M_valid, 1 = valid token, 0 = invalid, element-wise product;
 *     Algorithm 1, the migration step; Section 8, KV data must migrate).
 * The paper does not say what a layer computes.  The layer here is the
 * Llama-style pre-norm decoder layer (RMSNorm, rotary positions in the
 * rotate-half pairing, causal softmax attention with grouped KV heads, SwiGLU
 * feed-forward, two residual adds); that choice, and every other reading of a
 * point the paper leaves open, is listed in the design document.
 *
 * A second layer kind states the OPT-style decoder layer (the model family the
 * paper's own per-stage numbers are for, Table 2: OPT-66B): LayerNorm with bias
 * before each block, biased linear maps, no rotary embedding (positions enter
 * before the first layer, outside any stage), ReLU feed-forward.
 *
 * Precision: weights, inputs and cache contents arrive as float (the tests feed
 * values that are exactly representable in bf16); every intermediate is double;
 * nothing is rounded between operations.  The cache this oracle appends to is
 * float storage.
 *
 * Pins (tests with -m "not gpu"): RMSNorm closed forms; RoPE identity at
 * position 0, norm preservation, relative-position property; softmax rows sum
 * to one, one-key context returns V_0, equal keys give the mean of V; grouped
 * heads == replicated heads; library cross-checks (float64 matmul, float64
 * scaled-dot-product attention); an independent float64 re-statement of the
 * whole layer; split == unsplit; cached decode == recompute; repartition
 * against an independent index walk and brute force; incremental repartition:
 * snapshot pass + delta pass == one pass, rows outside the range untouched.
 *
 * Layouts (all row-major, last index fastest):
 *   weight matrices      [out_features][in_features]
 *   hidden               [token][hidden]
 *   kv pool              [layer - layer_begin][block][2: K,V][kv_head][slot][head_dim]
 *   block table          [sequence][max_blocks_per_seq]   (physical block ids)
 *   packed kv buffer     [sequence][layer - lb][logical block][2][kv_head][slot][head_dim]
 *   token-dense buffer   [sequence][layer - lb][2][kv_head][token - from_i][head_dim]
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* threads the parallel loops will use (for reporting the timed baseline) */
int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

typedef struct {
    int32_t hidden, n_q_heads, n_kv_heads, head_dim, ffn, kv_block_size;
    double rms_eps, rope_base;
} orc_shape;

typedef struct {
    const float *g_attn, *wq, *wk, *wv, *wo, *g_ffn, *w_gate, *w_up, *w_down;
} orc_layer;

typedef struct {
    void *base;                 /* pool memory of this stage                    */
    int64_t num_blocks;         /* physical blocks per layer in the pool        */
    int32_t layer_begin, layer_end; /* model layers [begin,end) the pool holds  */
    const int32_t *block_table; /* [num_seqs][max_blocks_per_seq]               */
    int32_t max_blocks_per_seq;
} orc_kv_view;

/* ------------------------------------------------------------------ */
/* elementary operations                                              */
/* ------------------------------------------------------------------ */

/* RMSNorm: y_k = x_k * g_k / sqrt(mean_k(x_k^2) + eps). */
void orc_rmsnorm(const double *x, const float *g, int32_t H, double eps, double *y)
{
    double ss = 0.0;
    for (int32_t k = 0; k < H; ++k) ss += x[k] * x[k];
    double r = 1.0 / sqrt(ss / (double)H + eps);
    for (int32_t k = 0; k < H; ++k) y[k] = x[k] * r * (double)g[k];
}

/* y[t][n] = sum_k W[n][k] * x[t][k]   for T rows of x. */
void orc_linear(const double *x, int32_t T, const float *W, int32_t N, int32_t K, double *y)
{
#pragma omp parallel for schedule(static)
    for (int32_t n = 0; n < N; ++n) {
        const float *w = W + (size_t)n * K;
        for (int32_t t = 0; t < T; ++t) {
            const double *xt = x + (size_t)t * K;
            double acc = 0.0;
            for (int32_t k = 0; k < K; ++k) acc += (double)w[k] * xt[k];
            y[(size_t)t * N + n] = acc;
        }
    }
}

/* Rotary position embedding of one head vector u[D] at absolute position pos,
 * rotate-half pairing: for d < D/2, angle = pos * base^(-2d/D),
 * (u_d, u_{d+D/2}) <- (u_d cos - u_{d+D/2} sin, u_{d+D/2} cos + u_d sin). */
void orc_rope(double *u, int32_t D, int64_t pos, double base)
{
    int32_t half = D / 2;
    for (int32_t d = 0; d < half; ++d) {
        double ang = (double)pos * pow(base, -2.0 * (double)d / (double)D);
        double c = cos(ang), s = sin(ang);
        double a = u[d], b = u[d + half];
        u[d] = a * c - b * s;
        u[d + half] = b * c + a * s;
    }
}

double orc_silu(double z) { return z / (1.0 + exp(-z)); }

/* In-place softmax over s[0..n): subtract the maximum, exponentiate, normalise. */
void orc_softmax(double *s, int32_t n)
{
    double m = s[0];
    for (int32_t r = 1; r < n; ++r) if (s[r] > m) m = s[r];
    double z = 0.0;
    for (int32_t r = 0; r < n; ++r) { s[r] = exp(s[r] - m); z += s[r]; }
    for (int32_t r = 0; r < n; ++r) s[r] /= z;
}

/* address of cache row (layer-local index ll, physical block pb, kv, head, slot) */
static inline size_t pool_row(const orc_shape *sh, int64_t num_blocks, int32_t ll,
                              int64_t pb, int32_t kv, int32_t head, int32_t slot)
{
    size_t bs = (size_t)sh->kv_block_size, D = (size_t)sh->head_dim, Hkv = (size_t)sh->n_kv_heads;
    return (((((size_t)ll * (size_t)num_blocks + (size_t)pb) * 2 + (size_t)kv) * Hkv + (size_t)head) * bs
            + (size_t)slot) * D;
}

/* Attention of ONE query token (all its heads) at absolute position p over the
 * keys 0..p of its sequence, read through the sequence's block-table row.
 *   q      [Hq][D]  (already rotated)
 *   o      [Hq][D]
 *   probs  optional [Hq][probs_stride]; entries 0..p are written
 * Query head h uses KV head h / (Hq/Hkv). */
void orc_attend_token(const orc_shape *sh, const float *pool, int64_t num_blocks, int32_t ll,
                      const int32_t *table_row, int64_t p, const double *q, double *o,
                      double *probs, int64_t probs_stride)
{
    int32_t D = sh->head_dim, Hq = sh->n_q_heads, Hkv = sh->n_kv_heads, bs = sh->kv_block_size;
    int32_t group = Hq / Hkv;
    int64_t n = p + 1;
    double *s = (double *)malloc(sizeof(double) * (size_t)n);
    for (int32_t h = 0; h < Hq; ++h) {
        int32_t hk = h / group;
        const double *qh = q + (size_t)h * D;
        for (int64_t r = 0; r < n; ++r) {
            const float *krow = pool + pool_row(sh, num_blocks, ll, table_row[r / bs], 0, hk, (int32_t)(r % bs));
            double acc = 0.0;
            for (int32_t d = 0; d < D; ++d) acc += qh[d] * (double)krow[d];
            s[r] = acc / sqrt((double)D);
        }
        orc_softmax(s, (int32_t)n);
        double *oh = o + (size_t)h * D;
        for (int32_t d = 0; d < D; ++d) oh[d] = 0.0;
        for (int64_t r = 0; r < n; ++r) {
            const float *vrow = pool + pool_row(sh, num_blocks, ll, table_row[r / bs], 1, hk, (int32_t)(r % bs));
            for (int32_t d = 0; d < D; ++d) oh[d] += s[r] * (double)vrow[d];
        }
        if (probs) for (int64_t r = 0; r < n; ++r) probs[(size_t)h * probs_stride + r] = s[r];
    }
    free(s);
}

/* ------------------------------------------------------------------ */
/* stage forward                                                      */
/* ------------------------------------------------------------------ */

/* Runs layers [0,n_layers) of `layers` (the stage's own layers, in order) over
 * one ragged batch.  Sequence i contributes tokens cu_seqlens_q[i] ..
 * cu_seqlens_q[i+1]-1; its j-th new token sits at absolute position
 * ctx_lens[i] + j, where ctx_lens[i] tokens are already in the cache.  The new
 * tokens' K (rotated) and V are appended to the pool; attention is causal.
 *   pool      float [n_layers][num_blocks][2][Hkv][bs][D], read and appended to
 *   hidden_in / hidden_out   double [T][H]
 *   probs     optional double [n_layers][T][Hq][probs_stride]
 * Returns 0, or -1 on a malformed argument. */
int orc_stage_forward(const orc_shape *sh, const orc_layer *layers, int32_t n_layers,
                      float *pool, int64_t num_blocks,
                      int32_t num_seqs, const int32_t *cu_seqlens_q, const int32_t *ctx_lens,
                      const int32_t *block_table, int32_t max_blocks_per_seq,
                      const double *hidden_in, double *hidden_out,
                      double *probs, int64_t probs_stride)
{
    int32_t H = sh->hidden, D = sh->head_dim, Hq = sh->n_q_heads, Hkv = sh->n_kv_heads;
    int32_t F = sh->ffn, bs = sh->kv_block_size;
    if (!sh || !layers || n_layers < 0 || num_seqs < 0 || Hkv <= 0 || Hq % Hkv || D % 2) return -1;
    int32_t T = num_seqs ? cu_seqlens_q[num_seqs] : 0;
    if (T == 0) return 0;
    for (int32_t i = 0; i < num_seqs; ++i) {
        int64_t after = (int64_t)ctx_lens[i] + (cu_seqlens_q[i + 1] - cu_seqlens_q[i]);
        if ((after + bs - 1) / bs > max_blocks_per_seq) return -1;
    }
    /* token -> (sequence, absolute position) */
    int32_t *tok_seq = (int32_t *)malloc(sizeof(int32_t) * (size_t)T);
    int64_t *tok_pos = (int64_t *)malloc(sizeof(int64_t) * (size_t)T);
    for (int32_t i = 0; i < num_seqs; ++i)
        for (int32_t t = cu_seqlens_q[i]; t < cu_seqlens_q[i + 1]; ++t) {
            tok_seq[t] = i;
            tok_pos[t] = (int64_t)ctx_lens[i] + (t - cu_seqlens_q[i]);
        }
    size_t TH = (size_t)T * H, TQ = (size_t)T * Hq * D, TK = (size_t)T * Hkv * D, TF = (size_t)T * F;
    double *x = (double *)malloc(sizeof(double) * TH);
    double *nrm = (double *)malloc(sizeof(double) * TH);
    double *q = (double *)malloc(sizeof(double) * TQ);
    double *k = (double *)malloc(sizeof(double) * TK);
    double *v = (double *)malloc(sizeof(double) * TK);
    double *o = (double *)malloc(sizeof(double) * TQ);
    double *proj = (double *)malloc(sizeof(double) * TH);
    double *hmid = (double *)malloc(sizeof(double) * TH);
    double *gate = (double *)malloc(sizeof(double) * TF);
    double *up = (double *)malloc(sizeof(double) * TF);
    memcpy(x, hidden_in, sizeof(double) * TH);

    for (int32_t ll = 0; ll < n_layers; ++ll) {
        const orc_layer *L = &layers[ll];
        /* 1. attention norm */
        for (int32_t t = 0; t < T; ++t) orc_rmsnorm(x + (size_t)t * H, L->g_attn, H, sh->rms_eps, nrm + (size_t)t * H);
        /* 2. q, k, v projections */
        orc_linear(nrm, T, L->wq, Hq * D, H, q);
        orc_linear(nrm, T, L->wk, Hkv * D, H, k);
        orc_linear(nrm, T, L->wv, Hkv * D, H, v);
        /* 3. rotary embedding of q and k;  4. append rotated k and raw v to the cache */
        for (int32_t t = 0; t < T; ++t) {
            int64_t p = tok_pos[t];
            const int32_t *row = block_table + (size_t)tok_seq[t] * max_blocks_per_seq;
            for (int32_t h = 0; h < Hq; ++h) orc_rope(q + ((size_t)t * Hq + h) * D, D, p, sh->rope_base);
            for (int32_t h = 0; h < Hkv; ++h) {
                double *kh = k + ((size_t)t * Hkv + h) * D;
                double *vh = v + ((size_t)t * Hkv + h) * D;
                orc_rope(kh, D, p, sh->rope_base);
                float *kdst = pool + pool_row(sh, num_blocks, ll, row[p / bs], 0, h, (int32_t)(p % bs));
                float *vdst = pool + pool_row(sh, num_blocks, ll, row[p / bs], 1, h, (int32_t)(p % bs));
                for (int32_t d = 0; d < D; ++d) { kdst[d] = (float)kh[d]; vdst[d] = (float)vh[d]; }
            }
        }
        /* 5. causal attention over keys 0..p */
#pragma omp parallel for schedule(dynamic, 1)
        for (int32_t t = 0; t < T; ++t) {
            const int32_t *row = block_table + (size_t)tok_seq[t] * max_blocks_per_seq;
            double *pr = probs ? probs + (((size_t)ll * T + t) * Hq) * (size_t)probs_stride : NULL;
            orc_attend_token(sh, pool, num_blocks, ll, row, tok_pos[t],
                             q + (size_t)t * Hq * D, o + (size_t)t * Hq * D, pr, probs_stride);
        }
        /* 6. output projection + residual */
        orc_linear(o, T, L->wo, H, Hq * D, proj);
        for (size_t e = 0; e < TH; ++e) hmid[e] = x[e] + proj[e];
        /* 7. feed-forward: norm, SwiGLU, down projection + residual */
        for (int32_t t = 0; t < T; ++t) orc_rmsnorm(hmid + (size_t)t * H, L->g_ffn, H, sh->rms_eps, nrm + (size_t)t * H);
        orc_linear(nrm, T, L->w_gate, F, H, gate);
        orc_linear(nrm, T, L->w_up, F, H, up);
        for (size_t e = 0; e < TF; ++e) gate[e] = orc_silu(gate[e]) * up[e];
        orc_linear(gate, T, L->w_down, H, F, proj);
        for (size_t e = 0; e < TH; ++e) x[e] = hmid[e] + proj[e];
    }
    memcpy(hidden_out, x, sizeof(double) * TH);
    free(tok_seq); free(tok_pos); free(x); free(nrm); free(q); free(k); free(v); free(o);
    free(proj); free(hmid); free(gate); free(up);
    return 0;
}

/* ------------------------------------------------------------------ */
/* KV repartition: exact data movement on elements of elem_bytes      */
/* ------------------------------------------------------------------ */

static const orc_kv_view *view_with_layer(const orc_kv_view *v, int32_t n, int32_t layer)
{
    for (int32_t s = 0; s < n; ++s)
        if (layer >= v[s].layer_begin && layer < v[s].layer_end) return &v[s];
    return NULL;
}

/* Both view lists must tile the same layer range without gaps or overlap. */
static int views_cover_same_range(const orc_kv_view *a, int32_t na, const orc_kv_view *b, int32_t nb)
{
    if (na <= 0 || nb <= 0) return 0;
    for (int32_t s = 0; s < na; ++s) if (a[s].layer_begin >= a[s].layer_end) return 0;
    for (int32_t s = 0; s < nb; ++s) if (b[s].layer_begin >= b[s].layer_end) return 0;
    for (int32_t s = 1; s < na; ++s) if (a[s].layer_begin != a[s - 1].layer_end) return 0;
    for (int32_t s = 1; s < nb; ++s) if (b[s].layer_begin != b[s - 1].layer_end) return 0;
    return a[0].layer_begin == b[0].layer_begin && a[na - 1].layer_end == b[nb - 1].layer_end;
}

/* For every destination stage, every layer it owns, every sequence i, every
 * valid token r < ctx_lens[i], K and V, every head: the token's row is copied
 * from where the source stage that owns the layer keeps it to where the
 * destination table puts it.  Slots r >= ctx_lens[i] inside the last touched
 * destination block are zero (the element-wise product with the validity mask
 * of Eq. 10).  Destination blocks no sequence maps to are left alone. */
int orc_kv_repartition(const orc_shape *sh, int32_t elem_bytes,
                       const orc_kv_view *src, int32_t n_src,
                       const orc_kv_view *dst, int32_t n_dst,
                       const int32_t *ctx_lens, int32_t num_seqs)
{
    if (!views_cover_same_range(src, n_src, dst, n_dst)) return -1;
    int32_t bs = sh->kv_block_size, D = sh->head_dim, Hkv = sh->n_kv_heads;
    size_t row_bytes = (size_t)D * (size_t)elem_bytes;
    for (int32_t d = 0; d < n_dst; ++d) {
        const orc_kv_view *dv = &dst[d];
        for (int32_t layer = dv->layer_begin; layer < dv->layer_end; ++layer) {
            const orc_kv_view *sv = view_with_layer(src, n_src, layer);
            if (!sv) return -1;
            for (int32_t i = 0; i < num_seqs; ++i) {
                int32_t c = ctx_lens[i];
                int32_t nblk = (c + bs - 1) / bs;
                if (nblk > sv->max_blocks_per_seq || nblk > dv->max_blocks_per_seq) return -1;
                const int32_t *srow = sv->block_table + (size_t)i * sv->max_blocks_per_seq;
                const int32_t *drow = dv->block_table + (size_t)i * dv->max_blocks_per_seq;
                for (int32_t r = 0; r < nblk * bs; ++r)
                    for (int32_t kv = 0; kv < 2; ++kv)
                        for (int32_t h = 0; h < Hkv; ++h) {
                            size_t so = pool_row(sh, sv->num_blocks, layer - sv->layer_begin, srow[r / bs], kv, h, r % bs);
                            size_t dof = pool_row(sh, dv->num_blocks, layer - dv->layer_begin, drow[r / bs], kv, h, r % bs);
                            unsigned char *dp = (unsigned char *)dv->base + dof * (size_t)elem_bytes;
                            if (r < c) memcpy(dp, (const unsigned char *)sv->base + so * (size_t)elem_bytes, row_bytes);
                            else memset(dp, 0, row_bytes);
                        }
            }
        }
    }
    return 0;
}

/* Number of elements in the packed buffer for layers [lb,le). */
int64_t orc_kv_packed_elems(const orc_shape *sh, int32_t lb, int32_t le,
                            const int32_t *ctx_lens, int32_t num_seqs)
{
    int64_t blocks = 0;
    for (int32_t i = 0; i < num_seqs; ++i) blocks += (ctx_lens[i] + sh->kv_block_size - 1) / sh->kv_block_size;
    return blocks * (int64_t)(le - lb) * 2 * sh->n_kv_heads * sh->kv_block_size * sh->head_dim;
}

/* pack: gather layers [lb,le) of one source view into the contiguous buffer
 * [sequence][layer-lb][logical block][2][kv_head][slot][head_dim], invalid
 * slots zero.  unpack: the inverse scatter into one destination view. */
static int pack_or_unpack(const orc_shape *sh, int32_t elem_bytes, const orc_kv_view *view,
                          int32_t lb, int32_t le, const int32_t *ctx_lens, int32_t num_seqs,
                          unsigned char *packed, int to_packed)
{
    if (lb < view->layer_begin || le > view->layer_end || lb >= le) return -1;
    int32_t bs = sh->kv_block_size, D = sh->head_dim, Hkv = sh->n_kv_heads;
    size_t row_bytes = (size_t)D * (size_t)elem_bytes;
    size_t cursor = 0; /* in rows of D elements */
    for (int32_t i = 0; i < num_seqs; ++i) {
        int32_t c = ctx_lens[i];
        int32_t nblk = (c + bs - 1) / bs;
        if (nblk > view->max_blocks_per_seq) return -1;
        const int32_t *row = view->block_table + (size_t)i * view->max_blocks_per_seq;
        for (int32_t layer = lb; layer < le; ++layer)
            for (int32_t j = 0; j < nblk; ++j)
                for (int32_t kv = 0; kv < 2; ++kv)
                    for (int32_t h = 0; h < Hkv; ++h)
                        for (int32_t slot = 0; slot < bs; ++slot, ++cursor) {
                            size_t po = pool_row(sh, view->num_blocks, layer - view->layer_begin, row[j], kv, h, slot);
                            unsigned char *pp = (unsigned char *)view->base + po * (size_t)elem_bytes;
                            unsigned char *bp = packed + cursor * row_bytes;
                            int valid = j * bs + slot < c;
                            if (to_packed) { if (valid) memcpy(bp, pp, row_bytes); else memset(bp, 0, row_bytes); }
                            else           { if (valid) memcpy(pp, bp, row_bytes); else memset(pp, 0, row_bytes); }
                        }
    }
    return 0;
}

int orc_kv_pack(const orc_shape *sh, int32_t elem_bytes, const orc_kv_view *src, int32_t lb, int32_t le,
                const int32_t *ctx_lens, int32_t num_seqs, void *packed)
{
    return pack_or_unpack(sh, elem_bytes, src, lb, le, ctx_lens, num_seqs, (unsigned char *)packed, 1);
}

int orc_kv_unpack(const orc_shape *sh, int32_t elem_bytes, const void *packed, const orc_kv_view *dst,
                  int32_t lb, int32_t le, const int32_t *ctx_lens, int32_t num_seqs)
{
    return pack_or_unpack(sh, elem_bytes, dst, lb, le, ctx_lens, num_seqs, (unsigned char *)packed, 0);
}

/* ---------------------------------------------------------------------------
 * Incremental repartition.  Section 6.3 lets the cache transfer run while
 * inference continues on the old configuration, so a first pass moves a
 * snapshot and later passes move what was appended since.  The validity mask of
 * Eq. 10 ("tokens that need synchronization") is then, per sequence i, the
 * token range [from_i, to_i):
 *   - every row of a token r with from_i <= r < to_i is copied as in
 *     orc_kv_repartition;
 *   - if the range is not empty, the slots r >= to_i of the block that holds
 *     token to_i - 1 are zero (the mask's zeros);
 *   - nothing else is written: rows of tokens r < from_i (moved by an earlier
 *     pass) and blocks outside the range keep their contents.
 * With from_i = 0 this is orc_kv_repartition. */
int orc_kv_repartition_range(const orc_shape *sh, int32_t elem_bytes,
                             const orc_kv_view *src, int32_t n_src,
                             const orc_kv_view *dst, int32_t n_dst,
                             const int32_t *from_lens, const int32_t *to_lens, int32_t num_seqs)
{
    if (!views_cover_same_range(src, n_src, dst, n_dst)) return -1;
    int32_t bs = sh->kv_block_size, D = sh->head_dim, Hkv = sh->n_kv_heads;
    size_t row_bytes = (size_t)D * (size_t)elem_bytes;
    for (int32_t i = 0; i < num_seqs; ++i)
        if (from_lens[i] < 0 || from_lens[i] > to_lens[i]) return -1;
    for (int32_t d = 0; d < n_dst; ++d) {
        const orc_kv_view *dv = &dst[d];
        for (int32_t layer = dv->layer_begin; layer < dv->layer_end; ++layer) {
            const orc_kv_view *sv = view_with_layer(src, n_src, layer);
            if (!sv) return -1;
            for (int32_t i = 0; i < num_seqs; ++i) {
                int32_t lo = from_lens[i], hi = to_lens[i];
                if (lo == hi) continue;
                int32_t nblk = (hi + bs - 1) / bs;
                if (nblk > sv->max_blocks_per_seq || nblk > dv->max_blocks_per_seq) return -1;
                const int32_t *srow = sv->block_table + (size_t)i * sv->max_blocks_per_seq;
                const int32_t *drow = dv->block_table + (size_t)i * dv->max_blocks_per_seq;
                for (int32_t r = lo; r < nblk * bs; ++r)
                    for (int32_t kv = 0; kv < 2; ++kv)
                        for (int32_t h = 0; h < Hkv; ++h) {
                            size_t so = pool_row(sh, sv->num_blocks, layer - sv->layer_begin, srow[r / bs], kv, h, r % bs);
                            size_t dof = pool_row(sh, dv->num_blocks, layer - dv->layer_begin, drow[r / bs], kv, h, r % bs);
                            unsigned char *dp = (unsigned char *)dv->base + dof * (size_t)elem_bytes;
                            if (r < hi) memcpy(dp, (const unsigned char *)sv->base + so * (size_t)elem_bytes, row_bytes);
                            else memset(dp, 0, row_bytes);
                        }
            }
        }
    }
    return 0;
}

/* Token-dense packed form of the same range: only the rows of tokens
 * [from_i, to_i), no padding to whole blocks, ordered
 * [sequence][layer - lb][K,V][kv_head][token - from_i][head_dim].
 * This is what a delta pass between devices would carry: a few tokens per
 * sequence, where the block-granular buffer would be mostly padding. */
int64_t orc_kv_packed_tokens_elems(const orc_shape *sh, int32_t lb, int32_t le,
                                   const int32_t *from_lens, const int32_t *to_lens, int32_t num_seqs)
{
    int64_t tokens = 0;
    for (int32_t i = 0; i < num_seqs; ++i) tokens += to_lens[i] - from_lens[i];
    return tokens * (int64_t)(le - lb) * 2 * sh->n_kv_heads * sh->head_dim;
}

/* to_packed: gather the rows into the buffer.  Otherwise: scatter them into the
 * view and zero the slots after to_i - 1 in its block, as the range repartition
 * does, so that pack followed by unpack equals orc_kv_repartition_range. */
static int pack_or_unpack_tokens(const orc_shape *sh, int32_t elem_bytes, const orc_kv_view *view,
                                 int32_t lb, int32_t le, const int32_t *from_lens, const int32_t *to_lens,
                                 int32_t num_seqs, unsigned char *packed, int to_packed)
{
    if (lb < view->layer_begin || le > view->layer_end || lb >= le) return -1;
    int32_t bs = sh->kv_block_size, D = sh->head_dim, Hkv = sh->n_kv_heads;
    size_t row_bytes = (size_t)D * (size_t)elem_bytes;
    for (int32_t i = 0; i < num_seqs; ++i)
        if (from_lens[i] < 0 || from_lens[i] > to_lens[i]) return -1;
    size_t cursor = 0; /* in rows of D elements */
    for (int32_t i = 0; i < num_seqs; ++i) {
        int32_t lo = from_lens[i], hi = to_lens[i];
        if (lo == hi) continue;
        int32_t nblk = (hi + bs - 1) / bs;
        if (nblk > view->max_blocks_per_seq) return -1;
        const int32_t *row = view->block_table + (size_t)i * view->max_blocks_per_seq;
        for (int32_t layer = lb; layer < le; ++layer)
            for (int32_t kv = 0; kv < 2; ++kv)
                for (int32_t h = 0; h < Hkv; ++h) {
                    for (int32_t r = lo; r < hi; ++r, ++cursor) {
                        size_t po = pool_row(sh, view->num_blocks, layer - view->layer_begin, row[r / bs], kv, h, r % bs);
                        unsigned char *pp = (unsigned char *)view->base + po * (size_t)elem_bytes;
                        unsigned char *bp = packed + cursor * row_bytes;
                        if (to_packed) memcpy(bp, pp, row_bytes); else memcpy(pp, bp, row_bytes);
                    }
                    if (!to_packed)
                        for (int32_t r = hi; r < nblk * bs; ++r) {
                            size_t po = pool_row(sh, view->num_blocks, layer - view->layer_begin, row[r / bs], kv, h, r % bs);
                            memset((unsigned char *)view->base + po * (size_t)elem_bytes, 0, row_bytes);
                        }
                }
    }
    return 0;
}

int orc_kv_pack_tokens(const orc_shape *sh, int32_t elem_bytes, const orc_kv_view *src, int32_t lb, int32_t le,
                       const int32_t *from_lens, const int32_t *to_lens, int32_t num_seqs, void *packed)
{
    return pack_or_unpack_tokens(sh, elem_bytes, src, lb, le, from_lens, to_lens, num_seqs, (unsigned char *)packed, 1);
}

int orc_kv_unpack_tokens(const orc_shape *sh, int32_t elem_bytes, const void *packed, const orc_kv_view *dst,
                         int32_t lb, int32_t le, const int32_t *from_lens, const int32_t *to_lens, int32_t num_seqs)
{
    return pack_or_unpack_tokens(sh, elem_bytes, dst, lb, le, from_lens, to_lens, num_seqs, (unsigned char *)packed, 0);
}

/* ------------------------------------------------------------------ */
/* OPT-style layer (Table 2's model family)                           */
/* ------------------------------------------------------------------ */

typedef struct {
    const float *ln1_g, *ln1_b, *wq, *bq, *wk, *bk, *wv, *bv, *wo, *bo;
    const float *ln2_g, *ln2_b, *w_fc1, *b_fc1, *w_fc2, *b_fc2;
} orc_opt_layer;

/* LayerNorm: y_k = (x_k - mean) / sqrt(var + eps) * g_k + b_k, var = mean((x - mean)^2). */
void orc_layernorm(const double *x, const float *g, const float *b, int32_t H, double eps, double *y)
{
    double mean = 0.0;
    for (int32_t k = 0; k < H; ++k) mean += x[k];
    mean /= (double)H;
    double var = 0.0;
    for (int32_t k = 0; k < H; ++k) var += (x[k] - mean) * (x[k] - mean);
    var /= (double)H;
    double r = 1.0 / sqrt(var + eps);
    for (int32_t k = 0; k < H; ++k) y[k] = (x[k] - mean) * r * (double)g[k] + (double)b[k];
}

/* y[t][n] = sum_k x[t][k] W[n][k] + bias[n] */
void orc_linear_bias(const double *x, int32_t T, const float *W, const float *bias, int32_t N, int32_t K, double *y)
{
    orc_linear(x, T, W, N, K, y);
    for (int32_t t = 0; t < T; ++t)
        for (int32_t n = 0; n < N; ++n) y[(size_t)t * N + n] += (double)bias[n];
}

double orc_relu(double z) { return z > 0.0 ? z : 0.0; }

/* One stage of OPT-style layers over a ragged batch; arguments and cache
 * handling as in orc_stage_forward (sh->rms_eps is the LayerNorm epsilon,
 * sh->rope_base is unused).  Per layer and token:
 *   n = LN(x; ln1)            q,k,v = W n + b        k, v appended to the cache
 *   o = causal softmax attention (scores scaled by 1/sqrt(D))
 *   h = x + Wo o + bo         m = LN(h; ln2)
 *   y = h + W2 relu(W1 m + b1) + b2 */
int orc_stage_forward_opt(const orc_shape *sh, const orc_opt_layer *layers, int32_t n_layers,
                          float *pool, int64_t num_blocks,
                          int32_t num_seqs, const int32_t *cu_seqlens_q, const int32_t *ctx_lens,
                          const int32_t *block_table, int32_t max_blocks_per_seq,
                          const double *hidden_in, double *hidden_out,
                          double *probs, int64_t probs_stride)
{
    if (!sh || !layers || n_layers < 0 || num_seqs < 0 || sh->n_kv_heads <= 0 || sh->n_q_heads % sh->n_kv_heads) return -1;
    int32_t H = sh->hidden, D = sh->head_dim, Hq = sh->n_q_heads, Hkv = sh->n_kv_heads;
    int32_t F = sh->ffn, bs = sh->kv_block_size;
    int32_t T = num_seqs ? cu_seqlens_q[num_seqs] : 0;
    if (T == 0) return 0;
    for (int32_t i = 0; i < num_seqs; ++i) {
        int64_t after = (int64_t)ctx_lens[i] + (cu_seqlens_q[i + 1] - cu_seqlens_q[i]);
        if ((after + bs - 1) / bs > max_blocks_per_seq) return -1;
    }
    int32_t *tok_seq = (int32_t *)malloc(sizeof(int32_t) * (size_t)T);
    int64_t *tok_pos = (int64_t *)malloc(sizeof(int64_t) * (size_t)T);
    for (int32_t i = 0; i < num_seqs; ++i)
        for (int32_t t = cu_seqlens_q[i]; t < cu_seqlens_q[i + 1]; ++t) {
            tok_seq[t] = i;
            tok_pos[t] = (int64_t)ctx_lens[i] + (t - cu_seqlens_q[i]);
        }
    size_t TH = (size_t)T * H, TQ = (size_t)T * Hq * D, TK = (size_t)T * Hkv * D, TF = (size_t)T * F;
    double *x = (double *)malloc(sizeof(double) * TH);
    double *nrm = (double *)malloc(sizeof(double) * TH);
    double *q = (double *)malloc(sizeof(double) * TQ);
    double *k = (double *)malloc(sizeof(double) * TK);
    double *v = (double *)malloc(sizeof(double) * TK);
    double *o = (double *)malloc(sizeof(double) * TQ);
    double *proj = (double *)malloc(sizeof(double) * TH);
    double *hmid = (double *)malloc(sizeof(double) * TH);
    double *act = (double *)malloc(sizeof(double) * TF);
    memcpy(x, hidden_in, sizeof(double) * TH);

    for (int32_t ll = 0; ll < n_layers; ++ll) {
        const orc_opt_layer *L = &layers[ll];
        for (int32_t t = 0; t < T; ++t) orc_layernorm(x + (size_t)t * H, L->ln1_g, L->ln1_b, H, sh->rms_eps, nrm + (size_t)t * H);
        orc_linear_bias(nrm, T, L->wq, L->bq, Hq * D, H, q);
        orc_linear_bias(nrm, T, L->wk, L->bk, Hkv * D, H, k);
        orc_linear_bias(nrm, T, L->wv, L->bv, Hkv * D, H, v);
        for (int32_t t = 0; t < T; ++t) {
            int64_t p = tok_pos[t];
            const int32_t *row = block_table + (size_t)tok_seq[t] * max_blocks_per_seq;
            for (int32_t h = 0; h < Hkv; ++h) {
                const double *kh = k + ((size_t)t * Hkv + h) * D, *vh = v + ((size_t)t * Hkv + h) * D;
                float *kdst = pool + pool_row(sh, num_blocks, ll, row[p / bs], 0, h, (int32_t)(p % bs));
                float *vdst = pool + pool_row(sh, num_blocks, ll, row[p / bs], 1, h, (int32_t)(p % bs));
                for (int32_t d = 0; d < D; ++d) { kdst[d] = (float)kh[d]; vdst[d] = (float)vh[d]; }
            }
        }
#pragma omp parallel for schedule(dynamic, 1)
        for (int32_t t = 0; t < T; ++t) {
            const int32_t *row = block_table + (size_t)tok_seq[t] * max_blocks_per_seq;
            double *pr = probs ? probs + (((size_t)ll * T + t) * Hq) * (size_t)probs_stride : NULL;
            orc_attend_token(sh, pool, num_blocks, ll, row, tok_pos[t],
                             q + (size_t)t * Hq * D, o + (size_t)t * Hq * D, pr, probs_stride);
        }
        orc_linear_bias(o, T, L->wo, L->bo, H, Hq * D, proj);
        for (size_t e = 0; e < TH; ++e) hmid[e] = x[e] + proj[e];
        for (int32_t t = 0; t < T; ++t) orc_layernorm(hmid + (size_t)t * H, L->ln2_g, L->ln2_b, H, sh->rms_eps, nrm + (size_t)t * H);
        orc_linear_bias(nrm, T, L->w_fc1, L->b_fc1, F, H, act);
        for (size_t e = 0; e < TF; ++e) act[e] = orc_relu(act[e]);
        orc_linear_bias(act, T, L->w_fc2, L->b_fc2, H, F, proj);
        for (size_t e = 0; e < TH; ++e) x[e] = hmid[e] + proj[e];
    }
    memcpy(hidden_out, x, sizeof(double) * TH);
    free(tok_seq); free(tok_pos); free(x); free(nrm); free(q); free(k); free(v); free(o);
    free(proj); free(hmid); free(act);
    return 0;
}
