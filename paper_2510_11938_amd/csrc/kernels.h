// Host-side declarations of the kernel launchers (one translation unit per
// kernel family).  Internal to the library; the public ABI is include/flexstage.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>

namespace fxp {

// ---------------------------------------------------------------- machine and tuning
// gfx950 is built from eight accelerator dies (XCDs) with an L2 each; workgroup i of a launch goes to die i % kXcds.
constexpr int kXcds = 8;
// Compute units of the current device (256 on MI355X), asked once from the runtime.
int device_cus();
// Launch-shape overrides for kernel experiments.  Only a -DFXP_TUNING build reads them from the environment; the
// normal build compiles the defaults in, so launch shapes -- and with them the low-order bits of a result -- depend
// on the shapes of a call alone.
inline int tuning_int(const char *name, int dflt)
{
#ifdef FXP_TUNING
    const char *v = getenv(name);
    return (v && *v) ? atoi(v) : dflt;
#else
    (void)name;
    return dflt;
#endif
}

// ---------------------------------------------------------------- KV mover
constexpr int kMaxMoveJobs = 8;

// One end of a move.  table != nullptr: a paged pool addressed through a block
// table; table == nullptr: the contiguous packed buffer.
struct KvMoveSide {
    char *base;
    const int32_t *table;        // [num_seqs][max_blocks_per_seq] or nullptr
    int64_t num_blocks;          // pool: physical blocks per layer
    int64_t limit_bytes;         // packed: size of the buffer (0 = unchecked)
    int32_t layer_base;          // model layer stored at index 0
    int32_t n_layers;            // packed: layers in the buffer
    int32_t max_blocks_per_seq;
    int32_t token_dense;         // 1: buffer of token rows [sequence][layer][K,V][head][token - from][dim]
};
struct KvMoveJob {
    KvMoveSide src, dst;
    int32_t layer_begin, layer_end;   // model layers this job moves
};
struct KvMoveArgs {
    KvMoveJob jobs[kMaxMoveJobs];
    const int32_t *from_lens;    // device [num_seqs] or nullptr (= 0): first token of each sequence to move
    const int32_t *to_lens;      // device [num_seqs]: one past the last valid token
    int64_t unit_bytes;          // bytes of one (layer, block): 2 * Hkv * 16 * D * 2
    int32_t n_jobs, num_seqs, head_dim;
};
hipError_t launch_kv_move(const KvMoveArgs &args, int grid, hipStream_t stream);
int kv_move_chunk_bytes();     // bytes of one work item

// ---------------------------------------------------------------- weights
// W[N][K] row-major bf16 -> packed[n_tile / 8][k_step][n_tile % 8][lane][8] (k zero-padded to k_steps*32):
// one MFMA row operand (16 rows x 32 k) is 1 KiB, and the eight 16-row tiles that the wavefronts of a
// workgroup multiply in the same k-step lie next to each other, so what a workgroup asks for at one
// time is one contiguous stretch (HBM serves that a few per cent faster than scattered 1-2 KiB runs).
constexpr int kPackGroup = 8;
// index, in 16-byte chunks, of lane 0 of the operand (tile nt, k-step ks) of a matrix with KS k-steps
__host__ __device__ inline int64_t packed_operand(int nt, int ks, int KS)
{
    return (((int64_t)(nt / kPackGroup) * KS + ks) * kPackGroup + nt % kPackGroup) * 64;
}
constexpr int kPackStepStride = kPackGroup * 64;      // chunks between consecutive k-steps of one tile
// half_tiles > 0 (the q and k matrices: head_dim / 32): inside every head of 2 * half_tiles row tiles the tiles of the
// first and the second half of the head dimension alternate (tile j of the first half -> 2j, of the second -> 2j + 1), so
// that the two values a rotary pair (d, d + head_dim/2) needs sit in the same lane of neighbouring accumulator tiles.
hipError_t launch_weight_pack(const void *src, int N, int K, void *dst, int k_steps,
                              int tile_offset, int tile_stride, int half_tiles, hipStream_t stream);
hipError_t launch_bias_pack(const void *src, int n, void *dst, int half_tiles, hipStream_t stream);   // a q or k bias, same order
// column of the q|k|v projection output that holds dim d of a q or k head starting at column head_col
__host__ __device__ inline int rotary_col(int head_col, int d, int head_dim)
{
    const int half_tiles = head_dim / 32, j = d / 16;
    const int jp = j < half_tiles ? 2 * j : 2 * (j - half_tiles) + 1;
    return head_col + jp * 16 + d % 16;
}

// ---------------------------------------------------------------- projections
struct SkinnyArgs {
    const uint16_t *W;     // packed weights
    const uint16_t *X;     // token rows [M][ldx] bf16
    float *P;              // partial sums [S][M][N]
    uint16_t *A;           // optional activation output, replaces P (S == 1): act 0 = SwiGLU over interleaved gate|up
                           // tiles -> [M][N/2] (even R); act 1 = relu(sum + bias) -> [M][N]
    const uint16_t *bias;  // act 1: bias [N] bf16
    int act;
    int M, N, K, KS, NT, ldx, S;   // KS = padded K / 32, NT = N / 16
    int R;                         // 16-row weight tiles per wavefront: 1, 2 or 4
    int U;                         // k-steps per register buffer: 1, 2, 4 or 8 (rounded down to what the shape allows)
    int NB;                        // register buffers in the ring: 2 or 4 (4 only where the registers allow it)
};
hipError_t launch_gemm_skinny(const SkinnyArgs &a, hipStream_t stream);

struct RopeArgs {
    const float *P;        // q|k|v partial sums [S][T][Nall], or nullptr
    const uint16_t *qkv;   // q|k|v bf16 [T][Nall] (when P == nullptr)
    const uint16_t *bias;  // optional q|k|v bias [Nall] bf16, added to the partial sums (P != nullptr only)
    uint16_t *q_out;       // rotated q [T][Hq*D] bf16
    uint16_t *pool;        // stage KV pool
    const int32_t *tok_seq, *tok_pos;   // from the rope table
    const int32_t *tok_row;             // from the rope table: the token's K row for kv head 0 inside a layer of the pool
    const float *cs, *sn;
    const int32_t *block_table;
    int64_t num_blocks;
    int T, S, max_blocks_per_seq, layer_local;
    int n_q_heads, n_kv_heads, head_dim;
};
// kEpiRope: the q|k|v projection finishes its own rows: (+ bias,) round to bf16, rotary embedding of the q and k heads at
// the token's position, q -> bf16 buffer, rotated k and raw v -> the token's slot of the paged cache (`rope`; P, qkv, S
// and bias of it are not used).  Only the wide tile has this epilogue: gemm_wide_applies() says whether a launch gets it.
enum { kEpiStore = 0, kEpiResidual = 1, kEpiSwiglu = 2, kEpiPartial = 3, kEpiRelu = 4, kEpiRope = 5 };
struct TiledArgs {
    const uint16_t *W;     // packed weights
    const uint16_t *X;     // token rows [M][ldx] bf16
    const uint16_t *R;     // residual [M][ldc] (kEpiResidual), may alias C
    uint16_t *C;           // output [M][ldc] bf16
    float *P;              // kEpiPartial: float partial sums [S][M][NT*16]
    const uint16_t *bias;  // optional bias [NT*16] bf16, added before the residual / activation (not for kEpiPartial, kEpiSwiglu)
    int M, K, KS, NT, ldx, ldc, epilogue;
    int S;                 // kEpiPartial: split-K factor (grid.y)
    int blk_m;             // set by the launcher (wide tile): token tiles per XCD super-block, 8, 4, 2 or 1 (weight tiles: 32 / blk_m)
    RopeArgs rope;         // kEpiRope
};
hipError_t launch_gemm_tiled(const TiledArgs &a, hipStream_t stream);
bool gemm_wide_applies(const TiledArgs &a);      // the launch would run on the 256 x 256 tile (shape fits and it is the faster one)

// ---------------------------------------------------------------- row-wise kernels
// b == nullptr: RMSNorm, n = x * rsqrt(mean(x^2) + eps) * g;  else LayerNorm, n = (x - mean) * rsqrt(var + eps) * g + b
hipError_t launch_rmsnorm(const void *x, const void *g, const void *b, void *out, int T, int H, float eps, hipStream_t stream);

struct ResidNormArgs {
    const uint16_t *x;     // residual input [T][H]
    const float *P;        // projection partial sums [S][T][H]
    uint16_t *h;           // x + proj, bf16 [T][H] (may alias x)
    const uint16_t *bias;  // bias of the projection [H], or nullptr
    const uint16_t *g;     // gain of the following norm, or nullptr
    const uint16_t *nb;    // bias of the following norm: LayerNorm when set, RMSNorm when nullptr
    uint16_t *n;           // normed output [T][H] (when g)
    int T, H, S;
    float eps;
};
hipError_t launch_resid_norm(const ResidNormArgs &a, hipStream_t stream);

struct SwigluArgs {
    const float *P;        // act 0: gate|up partial sums [S][T][2F], rows interleaved in 16-tiles; act 1: [S][T][F]
    uint16_t *out;         // [T][ld_out] bf16
    const uint16_t *bias;  // act 1: bias [F] bf16
    int T, F, S, ld_out;
    int act;               // 0: silu(gate) * up;  1: relu(sum + bias)
};
hipError_t launch_swiglu(const SwigluArgs &a, hipStream_t stream);

struct RopeTableArgs {
    const int32_t *cu_seqlens_q, *ctx_lens;
    int32_t *tok_seq, *tok_pos;   // [T]
    // [T] cache row of each token's K for kv head 0: (block_table[seq][pos / 16] * 2 * n_kv_heads) * 16 + pos % 16, in
    // rows of head_dim values inside one layer of the pool (V: + n_kv_heads * 16; head h: + h * 16); the same for every layer
    int32_t *tok_row;
    const int32_t *block_table;
    int max_blocks_per_seq, n_kv_heads;
    int32_t *blk_prefix;          // [num_seqs + 1] exclusive prefix of ceil((ctx+1)/16): the decode kernels' work cut
    float *cs, *sn;               // [T][D/2]
    int T, num_seqs, head_dim;
    float rope_base;
    int identity;                 // 1: no rotary embedding (cos = 1, sin = 0)
    int one_token_each;           // 1: a pure decode step (token t belongs to sequence t): no search through cu_seqlens_q
    // the first layer's attention norm rides in the same launch (one launch less per step); skipped when norm_x is null
    const uint16_t *norm_x, *norm_g, *norm_b;   // rows [T][norm_H], gain, optional LayerNorm bias
    uint16_t *norm_out;
    int norm_H;
    float norm_eps;
};
hipError_t launch_rope_table(const RopeTableArgs &a, hipStream_t stream);

hipError_t launch_qkv_rope_kvwrite(const RopeArgs &a, hipStream_t stream);

// ---------------------------------------------------------------- attention
constexpr int kDecodeWorkersPerCu = 8;    // wavefronts of the decode kernel per compute unit (half of it for grouped queries at head_dim 128)

struct DecodeAttnArgs {
    const uint16_t *q;     // [num_seqs][Hq][D] bf16 (rotated)
    const uint16_t *pool;
    const int32_t *ctx_lens, *block_table;
    const int32_t *cu_seqlens_q; // [num_seqs + 1]: a sequence with exactly one new token is a decode row, at token row cu[seq]
    const int32_t *blk_prefix;   // [num_seqs + 1] from the rope-table kernel (decode rows only)
    float *part_acc;       // [n_workers + num_seqs*Hkv][G][D]   one row group per piece
    float *part_ml;        // [n_workers + num_seqs*Hkv][G][2]
    uint16_t *out;         // [num_seqs][Hq*D] bf16
    float *dbg_scores;     // optional [num_seqs][Hq][dbg_stride]
    int64_t dbg_stride;
    int64_t num_blocks;
    int num_seqs, max_blocks_per_seq, n_workers, layer_local;   // n_workers: multiple of 4
    int n_q_heads, n_kv_heads, head_dim;
    int head_group;        // kv heads (= wavefronts) per worker: 4, 2 or 1, a divisor of n_kv_heads
    float scale_log2e;     // log2(e) / sqrt(D)
};
int decode_head_group(int n_kv_heads);
bool decode_attn_supported(int head_dim, int group);
hipError_t launch_attn_decode(const DecodeAttnArgs &a, hipStream_t stream);          // per-split partial results
hipError_t launch_attn_decode_combine(const DecodeAttnArgs &a, hipStream_t stream);  // merge of the splits

struct PrefillAttnArgs {
    const uint16_t *q;     // [T][Hq][D] bf16 (rotated)
    const uint16_t *pool;
    const int32_t *cu_seqlens_q, *ctx_lens, *block_table;
    uint16_t *out;         // [T][Hq*D] bf16
    float *dbg_scores;     // optional [T][Hq][dbg_stride]
    float *dbg_ml;         // optional [T][Hq][3]
    int64_t dbg_stride;
    int64_t num_blocks;
    int num_seqs, num_tokens, max_q_len, max_blocks_per_seq, layer_local;
    int n_q_heads, n_kv_heads, head_dim;
    int skip_single;       // 1: sequences with one new token are left to the decode kernels
    float scale_log2e;
    // a launch with few query tiles cuts the keys of each tile into up to kv_split pieces (prefill_kv_split) and merges them
    const int32_t *tok_seq;      // [T] sequence of each token (from the rope table)
    float *part_acc;             // [kv_split][T][Hq][D] unnormalised sums of the pieces; nullptr: never cut
    float *part_ml;              // [kv_split][T][Hq][2] running maximum (log2 domain) and denominator
    int kv_split;
    int q_tile;                  // query rows per workgroup: 64 or 128 (prefill_q_tile)
};
int prefill_q_tile(int n_q_heads, int num_tokens, int num_seqs, int max_q_len, int max_blocks_per_seq);
int prefill_kv_split(int n_q_heads, int num_tokens, int num_seqs, int max_blocks_per_seq, int q_tile);
size_t prefill_piece_rows(int n_q_heads, int max_tokens);     // rows of part_acc / part_ml for calls of up to max_tokens
hipError_t launch_attn_prefill(const PrefillAttnArgs &a, hipStream_t stream);

}  // namespace fxp
