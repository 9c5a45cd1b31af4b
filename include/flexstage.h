/*
 * flexstage — C ABI of the MI355X (gfx950) stage-forward and KV-repartition library.
 *
 * The library executes the GPU work of ONE fine-grained pipeline stage of the
 * FlexPipe serving method: the forward step of a contiguous decoder-layer range
 * over a dynamic batch, and the movement of the stage's per-layer KV cache when
 * inflight refactoring merges or splits stage boundaries.
 *
 * General conventions
 *   - Every function returns FXP_OK (0) or a negative FXP_E* code; after a
 *     failure fxp_last_error() holds a message (thread-local, static storage).
 *     No exception or abort crosses this boundary.
 *   - Pointers marked DEVICE are HIP device pointers owned by the caller; the
 *     library borrows them for the duration of the call (the weight arena: for
 *     the life of the stage handle).  Pointers marked HOST are ordinary host
 *     memory.  The library allocates no device memory, ever.
 *   - All GPU work is enqueued on `hip_stream` (a hipStream_t passed as void*,
 *     NULL = the default stream) and the call returns without synchronising.
 *   - Host-side arguments are validated; the CONTENTS of device-side tables
 *     (block ids, lengths) are trusted and must be consistent with the sizes
 *     given on the host side.
 *   - bf16 = the 16-bit brain-float format (1 sign, 8 exponent, 7 mantissa bits).
 *   - Results are deterministic: the same inputs give bit-identical outputs,
 *     independent of the physical block placement and of how many layers the
 *     stage holds.  Launch shapes are fixed by the shapes of a call and the
 *     device's compute-unit count; no environment variable changes them.
 */
#ifndef FLEXSTAGE_H
#define FLEXSTAGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FXP_OK       0
#define FXP_EINVAL  (-1)   /* null pointer, bad layer range, unsupported shape            */
#define FXP_ENOSPC  (-2)   /* workspace, weight arena or packed buffer too small           */
#define FXP_EHIP    (-3)   /* a HIP call or kernel launch failed                           */

/* Sequences per call (batch of a forward step, sequence list of a repartition): the
 * kernels keep per-sequence prefix sums in LDS.  More than this is FXP_EINVAL. */
#define FXP_MAX_SEQS 4096

typedef struct fxp_stage fxp_stage;           /* opaque, library-owned host object */

/* A stage is a contiguous subset of the model's layers (Section 5: each stage
 * S_k is a subset of operators, the stages are disjoint and cover the graph). */
typedef struct {
    int32_t layer_begin, layer_end;           /* [l0, l1) in model numbering, l0 < l1   */
    int32_t hidden;                           /* H, multiple of 16                       */
    int32_t n_q_heads, n_kv_heads;            /* n_q_heads % n_kv_heads == 0             */
    int32_t head_dim;                         /* D: 64 or 128                            */
    int32_t ffn;                              /* F, multiple of 16                       */
    float   rms_eps;
    float   rope_base;
    int32_t kv_block_size;                    /* tokens per cache block: must be 16      */
    int32_t arch;                             /* FXP_ARCH_LLAMA or FXP_ARCH_OPT          */
} fxp_stage_desc;

/* Layer kinds.  LLAMA: RMSNorm, rotary embedding, SwiGLU feed-forward, no biases.
 * OPT (the model family of the paper's per-stage measurements, Table 2):
 * LayerNorm with bias (rms_eps is its epsilon), biased projections, no rotary
 * embedding (positions enter before the first layer, outside any stage; rope_base
 * is ignored), feed-forward relu(W1 m + b1) then W2 . + b2. */
#define FXP_ARCH_LLAMA 0
#define FXP_ARCH_OPT   1

/* One decoder layer's parameters.  DEVICE, bf16, every matrix row-major
 * [out_features][in_features]; gains are [hidden]. */
typedef struct {
    const void *g_attn;                       /* [H]            attention RMSNorm gain   */
    const void *wq, *wk, *wv;                 /* [Hq*D][H], [Hkv*D][H], [Hkv*D][H]       */
    const void *wo;                           /* [H][Hq*D]                               */
    const void *g_ffn;                        /* [H]            feed-forward RMSNorm gain*/
    const void *w_gate, *w_up;                /* [F][H]                                  */
    const void *w_down;                       /* [H][F]                                  */
    /* FXP_ARCH_OPT only (ignored for FXP_ARCH_LLAMA): w_gate must be NULL, w_up is the
     * first and w_down the second feed-forward matrix, g_attn / g_ffn are the LayerNorm
     * gains, and these biases are added: */
    const void *b_attn_norm, *b_ffn_norm;     /* [H]            LayerNorm biases         */
    const void *bq, *bk, *bv;                 /* [Hq*D], [Hkv*D], [Hkv*D]                */
    const void *bo;                           /* [H]                                     */
    const void *b_up;                         /* [F]                                     */
    const void *b_down;                       /* [H]                                     */
} fxp_layer_weights;

/* A stage's paged KV cache.  DEVICE, bf16, caller-owned, logical shape
 *   [layer - layer_begin][block][2: K,V][n_kv_heads][kv_block_size][head_dim].
 * K rows are stored after the rotary embedding. */
typedef struct {
    void   *base;
    int64_t num_blocks;                       /* physical blocks per layer               */
    int32_t layer_begin, layer_end;           /* model layers the pool holds             */
} fxp_kv_pool;

/* One step's dynamic batch (Section 7: stages serve dynamically batched
 * requests).  Sequence i contributes the tokens cu_seqlens_q[i] ..
 * cu_seqlens_q[i+1]-1 of the packed hidden matrix; its j-th new token has
 * absolute position ctx_lens[i] + j; ctx_lens[i] tokens are already cached.
 * Row i of the block table lists the physical blocks of sequence i and must
 * have room for ctx_lens[i] + q_len_i tokens.  One table per stage, shared by
 * the stage's layers. */
typedef struct {
    int32_t num_seqs;
    int32_t num_tokens;                       /* T = cu_seqlens_q[num_seqs]              */
    int32_t max_q_len;                        /* max over i of q_len_i (1 for decode)    */
    int32_t max_blocks_per_seq;               /* row pitch of block_table                */
    const int32_t *cu_seqlens_q;              /* DEVICE [num_seqs + 1]                   */
    const int32_t *ctx_lens;                  /* DEVICE [num_seqs]                       */
    const int32_t *block_table;               /* DEVICE [num_seqs][max_blocks_per_seq]   */
    int32_t min_q_len;                        /* min over i of q_len_i, or 0 = not known.  A hint only: the lengths
                                                 live on the device, so a ragged call launches the decode-attention
                                                 kernels for its single-token sequences unless this says there are
                                                 none (>= 2).  A wrong value costs time, never correctness.        */
} fxp_batch;

/* A stage's cache as seen by the repartition calls: pool + that stage's table. */
typedef struct {
    const fxp_kv_pool *pool;                  /* HOST pointer to the pool descriptor     */
    const int32_t *block_table;               /* DEVICE [num_seqs][max_blocks_per_seq]   */
    int32_t max_blocks_per_seq;
} fxp_kv_view;

/* ---- stage lifetime -------------------------------------------------------
 * Section 5 asks that the parameters of one logical group stay contiguous in
 * memory so that merged or split stages reuse the layout.  fxp_stage_create
 * therefore re-tiles each layer's matrices into ONE contiguous per-layer
 * record inside `weight_arena` (DEVICE, caller-owned, at least
 * fxp_stage_weight_arena_bytes(desc) bytes, 256-byte aligned); a stage
 * covering any sub-range of layers can point into the same arena.
 * `layers` is a HOST array of layer_end - layer_begin entries.  The packing
 * kernels run on `hip_stream`; the caller's source tensors may be released once
 * that work has completed, the arena must outlive the handle. */
size_t fxp_stage_weight_arena_bytes(const fxp_stage_desc *desc);
int    fxp_stage_create(const fxp_stage_desc *desc, const fxp_layer_weights *layers,
                        void *weight_arena, size_t weight_arena_bytes, void *hip_stream,
                        fxp_stage **out);
int    fxp_stage_destroy(fxp_stage *stage);

/* ---- refinement and consolidation of stages (Section 6: a stage is split when
 * burst capacity is needed and stages are merged in stable periods; Section 5:
 * the parameters of a group stay contiguous so that merged stages reuse the
 * existing layout).  Both calls are host-only metadata operations: the new
 * handles point into the arena of the stages they came from, no weight is
 * moved and nothing is enqueued on any stream.  The inputs stay valid and are
 * destroyed separately; the arena must outlive every handle that points into it.
 * split: layer_mid strictly inside the stage's range, else FXP_EINVAL.
 * merge: `upper` must start at the layer where `lower` ends, have the same model
 * geometry, and its layer records must directly follow `lower`'s in memory (true
 * for the halves of a split, or for stages created side by side in one arena);
 * otherwise FXP_EINVAL and the caller builds the merged stage with
 * fxp_stage_create.  fxp_stage_layers reports a handle's layer range. */
int    fxp_stage_split(const fxp_stage *stage, int32_t layer_mid, fxp_stage **lower, fxp_stage **upper);
int    fxp_stage_merge(const fxp_stage *lower, const fxp_stage *upper, fxp_stage **out);
int    fxp_stage_layers(const fxp_stage *stage, int32_t *layer_begin, int32_t *layer_end);

/* ---- stage forward (Section 3.2, Table 2 "Compute": per-stage inference) ---
 * hidden_out = layers [l0,l1) applied to hidden_in, both DEVICE bf16
 * [num_tokens][hidden] (they may be the same buffer).  Each layer is the
 * pre-norm decoder layer: RMSNorm, q/k/v projections, rotary embedding
 * (rotate-half pairing), append of K,V to the paged cache, causal softmax
 * attention over the cached prefix plus the new tokens, output projection +
 * residual, RMSNorm, SwiGLU feed-forward + residual.  The pool's layer range
 * must equal the stage's.  Any mix of sequences is one call: decode rows (one
 * new token), whole prompts, prompt chunks behind a cached prefix.  Low-order
 * bits of the result may depend on the host-side bounds of the call (token and
 * sequence counts, table width), which select tile shapes, never on where the
 * blocks lie.  `workspace` is DEVICE scratch of at least
 * fxp_stage_workspace_bytes(...) bytes for the given bounds, 256-byte aligned;
 * its contents are undefined afterwards. */
size_t fxp_stage_workspace_bytes(const fxp_stage *stage, int32_t max_tokens, int32_t max_seqs,
                                 int32_t max_blocks_per_seq);
int    fxp_stage_forward(fxp_stage *stage, const fxp_kv_pool *pool, const fxp_batch *batch,
                         const void *hidden_in, void *hidden_out,
                         void *workspace, size_t workspace_bytes, void *hip_stream);

/* The same step for callers that cannot allocate device memory or size a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation): the
 * workspace is a file-scope device array of FXP_STATIC_SCRATCH_BYTES inside the library,
 * which every GPU the library runs on holds until the process ends.  No device or pinned
 * memory is allocated or freed by this call, ever.  Arguments, kernels and results are
 * those of fxp_stage_forward (bit-identical for the same inputs).  A step whose bounds
 * need more than the static array (fxp_stage_workspace_bytes > FXP_STATIC_SCRATCH_BYTES:
 * long prefill chunks) is FXP_ENOSPC and nothing is enqueued.  The first call on a device
 * looks the array's device address up (once per device; do it outside a graph capture).
 * All calls on one GPU share the one array, whose contents are undefined between calls:
 * calls that overlap on one GPU (two streams, two threads) race; serialise them. */
#define FXP_STATIC_SCRATCH_BYTES (128u << 20)
int    fxp_stage_forward_static(fxp_stage *stage, const fxp_kv_pool *pool, const fxp_batch *batch,
                                const void *hidden_in, void *hidden_out, void *hip_stream);

/* Test-only variant: additionally writes the attention probabilities the
 * kernels computed, DEVICE float [n_layers][num_tokens][n_q_heads][probs_stride],
 * entries 0..position of each token (the rest is left untouched).  Meant for
 * small shapes. */
int    fxp_stage_forward_debug(fxp_stage *stage, const fxp_kv_pool *pool, const fxp_batch *batch,
                               const void *hidden_in, void *hidden_out,
                               void *workspace, size_t workspace_bytes,
                               float *probs, int64_t probs_stride, void *hip_stream);

/* ---- KV repartition (Section 6.3, Eq. 10; Algorithm 1, migration step) -----
 * When stage boundaries move, the cache of every layer moves to the stage that
 * now owns the layer, multiplied element-wise by the token validity mask: for
 * every destination view d, layer l in its range, sequence i, logical block
 * j < ceil(ctx_lens[i]/16): the K and V block is copied from the source view
 * that holds layer l (block src_table[i][j]) to dst_table_d[i][j]; slots at or
 * beyond ctx_lens[i] arrive as zero; destination blocks that no listed
 * sequence maps to are not written.  Bit-exact on the 16-bit words.
 * `src` and `dst` are HOST arrays; each list must tile the same layer range in
 * ascending order without gaps; source and destination pools must not overlap.
 * ctx_lens: DEVICE [num_seqs], the tokens valid after the last completed step.
 * Only desc->n_kv_heads, head_dim and kv_block_size are read. */
int    fxp_kv_repartition(const fxp_stage_desc *desc,
                          const fxp_kv_view *src, int32_t n_src,
                          const fxp_kv_view *dst, int32_t n_dst,
                          const int32_t *ctx_lens, int32_t num_seqs, void *hip_stream);

/* The two halves of a repartition that crosses devices (Section 8: the cache moves between
 * GPU devices over a network transfer; Section 6.3, Eq. 10 fixes WHAT arrives: the source
 * cache times the token validity mask).  Each half applies that rule on its side of the
 * transfer, so unpack(pack(src)) leaves exactly what fxp_kv_repartition leaves.  pack gathers layers
 * [layer_begin, layer_end) of ONE source view into a contiguous DEVICE buffer
 *   [sequence][layer - layer_begin][logical block][2: K,V][kv_head][slot][head_dim]
 * (invalid slots zero); unpack scatters such a buffer into ONE destination
 * view through its own table.  fxp_kv_packed_bytes computes the buffer size
 * from lengths in HOST memory.  pack/unpack read the lengths on the device and
 * cannot know the total on the host: `packed_bytes` is the size of the buffer
 * the caller really has, and a (layer, block) unit that would not lie wholly
 * inside it is skipped, so neither call ever touches memory past the buffer;
 * FXP_ENOSPC is returned only when not even one block per layer fits. */
/* fxp_kv_packed_bytes: sum over sequences of ceil(ctx_lens[i]/16) blocks x layers x one (layer, block)
 * unit of 2 * n_kv_heads * 16 * head_dim bf16 values: the valid blocks of Eq. 10's mask, whole blocks. */
size_t fxp_kv_packed_bytes(const fxp_stage_desc *desc, int32_t layer_begin, int32_t layer_end,
                           const int32_t *ctx_lens_host, int32_t num_seqs);
/* fxp_kv_pack (source side of Eq. 10): block j of sequence i, layer l goes from src_table[i][j] to its place in
 * the buffer; slots at or beyond ctx_lens[i] are written as zero. */
int    fxp_kv_pack(const fxp_stage_desc *desc, const fxp_kv_view *src,
                   int32_t layer_begin, int32_t layer_end,
                   const int32_t *ctx_lens, int32_t num_seqs,
                   void *packed, size_t packed_bytes, void *hip_stream);
/* fxp_kv_unpack (destination side of Eq. 10): the buffer's blocks go to dst_table[i][j] of the fresh table;
 * blocks that no listed sequence maps to are not written. */
int    fxp_kv_unpack(const fxp_stage_desc *desc, const void *packed, size_t packed_bytes,
                     const fxp_kv_view *dst, int32_t layer_begin, int32_t layer_end,
                     const int32_t *ctx_lens, int32_t num_seqs, void *hip_stream);

/* ---- incremental repartition --------------------------------------------------
 * Section 6.3 lets the cache transfer run while inference continues on the old
 * configuration: a first pass moves a snapshot, later passes move what decoding
 * appended meanwhile.  The validity mask of Eq. 10 is then, per sequence i, the
 * token range [from_lens[i], to_lens[i]):
 *   - the K and V rows of every token in the range are copied as above;
 *   - if the range is not empty, the slots at or beyond to_lens[i] in the block
 *     of token to_lens[i] - 1 arrive as zero;
 *   - nothing else is written: rows of tokens before from_lens[i] and all other
 *     blocks keep their contents.  A sequence with from >= to (or from < 0)
 *     moves nothing.
 * A pass over [0, c) followed by a pass over [c, c') leaves exactly what one
 * pass over [0, c') leaves.  from_lens, to_lens: DEVICE [num_seqs].  All other
 * arguments, errors and the no-overlap rule are those of fxp_kv_repartition,
 * which is this call with from_lens = 0. */
int    fxp_kv_repartition_range(const fxp_stage_desc *desc,
                                const fxp_kv_view *src, int32_t n_src,
                                const fxp_kv_view *dst, int32_t n_dst,
                                const int32_t *from_lens, const int32_t *to_lens,
                                int32_t num_seqs, void *hip_stream);

/* Token-dense halves of an incremental pass that crosses devices: only the rows
 * of the tokens in the range, without padding to whole blocks,
 *   [sequence][layer - layer_begin][2: K,V][kv_head][token - from_lens[i]][head_dim]
 * (a delta pass carries a few tokens per sequence, where the block-granular
 * buffer would be mostly padding).  unpack also zeroes the slots after token
 * to_lens[i] - 1 in its block, so pack + unpack equals fxp_kv_repartition_range.
 * fxp_kv_packed_tokens_bytes computes the size from lengths in HOST memory;
 * as for fxp_kv_pack, `packed_bytes` is the size the caller really has and no
 * call touches memory past it (rows that do not fit are skipped on both
 * sides); FXP_ENOSPC only if packed_bytes < 16. */
size_t fxp_kv_packed_tokens_bytes(const fxp_stage_desc *desc, int32_t layer_begin, int32_t layer_end,
                                  const int32_t *from_lens_host, const int32_t *to_lens_host, int32_t num_seqs);
int    fxp_kv_pack_tokens(const fxp_stage_desc *desc, const fxp_kv_view *src,
                          int32_t layer_begin, int32_t layer_end,
                          const int32_t *from_lens, const int32_t *to_lens, int32_t num_seqs,
                          void *packed, size_t packed_bytes, void *hip_stream);
int    fxp_kv_unpack_tokens(const fxp_stage_desc *desc, const void *packed, size_t packed_bytes,
                            const fxp_kv_view *dst, int32_t layer_begin, int32_t layer_end,
                            const int32_t *from_lens, const int32_t *to_lens, int32_t num_seqs,
                            void *hip_stream);

/* ---- granularity controller (host only; nothing is enqueued) ------------------
 * The scalar decision formulas of the method, to be fed with stage throughput
 * and latency measured through fxp_stage_forward at the candidate stage depths.
 * All pointers are HOST memory.
 *   fxp_ctl_cv                   nu_t = sigma_t / mu_t of the request arrival
 *                                intervals (Section 6; population deviation).
 *   fxp_ctl_select_granularity   Eq. 4: score_k = [alpha T_k/T_max + (1-alpha)
 *                                L_min/L_k] exp(-|nu_t - nu_k| / sigma) with T_max,
 *                                L_min over the candidates; *best_out = arg max
 *                                (lowest index on ties); scores_out[n_cand] may
 *                                be NULL.
 *   fxp_ctl_parallel_instances   Eq. 5: floor(capacity_total / (T_k / (beta1 +
 *                                beta2 eta_k))); -1 on a bad argument.
 *   fxp_ctl_multiplexing_penalty gamma(CV) = gamma0 (1 + alpha CV^2), Section 6.2.
 *   fxp_ctl_scaling_granularity  Eq. 11: floor(G_max / (1 + beta exp(-gamma cv
 *                                min(q/Q_max, 1)))); -1 on a bad argument.
 *   fxp_ctl_slo_satisfied        Section 7: 1 if (deadline - init_time) *
 *                                sum_k stage_throughput[k] / queue_len >=
 *                                requests, 0 if not, FXP_EINVAL on a bad argument.
 * The constants alpha, sigma, nu_k, beta, gamma are not published: parameters. */
typedef struct {
    int32_t n_stages;      /* eta_k */
    int32_t batch;         /* b_k   */
    double  throughput;    /* T_k, any unit, > 0 */
    double  latency;       /* L_k, any unit, > 0 */
    double  cv_opt;        /* nu_k: the CV this granularity suits best */
} fxp_granularity;
int     fxp_ctl_cv(const double *intervals, int32_t n, double *cv_out);
int     fxp_ctl_select_granularity(const fxp_granularity *cand, int32_t n_cand, double cv_now, double alpha,
                                   double sigma, double *scores_out, int32_t *best_out);
int64_t fxp_ctl_parallel_instances(double capacity_total, double throughput, double beta1, double beta2,
                                   int32_t n_stages);
double  fxp_ctl_multiplexing_penalty(double gamma0, double alpha, double cv);
int32_t fxp_ctl_scaling_granularity(int32_t g_max, double beta, double gamma, double cv, double queue_len,
                                    double queue_cap);
int     fxp_ctl_slo_satisfied(double deadline, double init_time, const double *stage_throughput, int32_t n_stages,
                              double queue_len, double requests);

/* ---- per-kernel timing for benchmarks ---------------------------------------
 * While enabled, every kernel launch the library makes is bracketed by a pair
 * of HIP events recorded on the caller's stream (up to 8192 launches; later
 * ones are not timed).  fxp_profile_enable(on) also clears what was recorded.
 * fxp_profile_read waits for the recorded events and returns the summed
 * duration and the launch count of one kernel class; classes are numbered
 * 0 .. fxp_profile_num_classes()-1 and named by fxp_profile_class_name.
 * Not thread-safe; the events perturb the stream slightly, so whole-step
 * throughput is measured with profiling off. */
int         fxp_profile_enable(int on);
int         fxp_profile_num_classes(void);
const char *fxp_profile_class_name(int kernel_class);
int         fxp_profile_read(int kernel_class, double *total_ms, int64_t *launches);
/* One recorded launch, in launch order; FXP_EINVAL once index is past the last record. */
int         fxp_profile_read_launch(int index, int *kernel_class, double *ms);

const char *fxp_last_error(void);
const char *fxp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FLEXSTAGE_H */
