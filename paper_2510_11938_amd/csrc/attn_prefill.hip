// Chunked-prefill attention over the paged cache: every new token of a sequence
// attends causally to the cached prefix plus the new tokens up to itself (all of
// which rope_kvwrite has already stored in the cache), flash-style with an
// online softmax so no score matrix is materialised.
//
// This is a dense contraction, so both products run on the matrix cores
// (v_mfma_f32_16x16x32_bf16), arranged so that no register shuffling is needed
// between them:
//   S^T[kv][q] = K[kv][:] . Q[q][:]      row operand K, column operand Q;
//                                         the accumulator leaves each lane with
//                                         4 consecutive kv of ONE query column;
//   softmax over kv per query column: 4 in-lane values + 2 cross-lane steps;
//   O^T[dim][q] += V^T[dim][kv] . P^T[kv][q]
//                                         P^T in accumulator layout is already
//                                         the column operand of the next MFMA
//                                         (k slots 8c..8c+7 of lane group c are
//                                         kv 4c..4c+3 of two 16-key sub-tiles);
//                                         V^T comes from the row-major V tile in
//                                         LDS through the transpose load
//                                         (ds_read_b64_tr_b16).
// A workgroup is 4 waves x 16 or 32 query rows (one or two column blocks per
// wave) of one (sequence, query head); the 64-key K and V tiles are staged once
// in LDS and shared by the 4 waves.  With two column blocks every K and V
// operand read from LDS feeds two MFMAs and a tile is staged once per 128 rows.
// Probabilities enter the second product rounded to bf16; everything else is
// float.  Rows of V past the sequence end are zeroed while staging so that a
// zero probability never meets an uninitialised (possibly NaN) value.
#include "kernels.h"
#include "common.hip.h"
#include <stdlib.h>
#include <math.h>
#include <algorithm>

namespace fxp {

constexpr int kPfThreads = 256;
constexpr int kPfKvTile = 64;       // keys per LDS tile (4 cache blocks)
constexpr int kPfMinPieceTiles = 8; // a query tile's keys are cut into pieces of at least this many LDS tiles
constexpr int kPfMaxPieces = 8;
// workgroups of this kernel that the chip holds at a time: 3 per compute unit with 64 query rows, 2 with 128
static int prefill_resident_wgs(int q_tile) { return (q_tile == 64 ? 3 : 2) * device_cus(); }

// Pieces that the keys of one query tile are cut into when the launch has too few query tiles to fill the chip (a short
// chunk behind a long cached prefix): as many as the launch allows, each at least kPfMinPieceTiles tiles long.
// The attention kernel and the merge kernel both derive it from the same lengths.
__device__ inline int kv_pieces(int n_tiles, int kv_split)
{
    return min(kv_split, max(1, n_tiles / kPfMinPieceTiles));
}

template <int D, int QB, bool DEBUG, bool FLAT>
__global__ __launch_bounds__(kPfThreads) void attn_prefill_kernel(PrefillAttnArgs a)
{
    constexpr int QW = 16 * QB;                   // query rows per wave
    constexpr int QT = 4 * QW;                    // query rows per workgroup
    constexpr int KS = D / 32;                    // k-steps of the QK product
    constexpr int DT = D / 16;                    // 16-dim tiles of the output
    constexpr int kKPitch = D * 2 + 16;           // bytes per K row in LDS (conflict-free 16-byte reads)
    constexpr int kVPitch = D * 2 + 32;           // bytes per V row in LDS: 8 rows land in 8 distinct 32-byte bank groups
    typedef short v4s __attribute__((ext_vector_type(4)));
    __shared__ __attribute__((aligned(16))) char s_k[kPfKvTile * kKPitch];
    __shared__ __attribute__((aligned(16))) char s_v[kPfKvTile * kVPitch];

    // Workgroups are launched in index order and a causal tile's work grows with its position in the sequence:
    // heads vary fastest, then sequences, and the tiles are taken from the last one of every sequence down, so
    // the long tiles of all sequences start first and the short ones fill the tail of the launch.
    int seq, t0, q_len, qt;
    const int h = blockIdx.x;
    // the tile index (from the last one down) and the piece share the slowest grid dimension that is used
    const int slow = FLAT ? (int)blockIdx.y : (int)blockIdx.z;
    const int piece = slow % a.kv_split, by = slow / a.kv_split;
    if constexpr (FLAT) {
        // Query tiles of all sequences as one line: sequence i owns the slots from cu[i] / QT + i on (cu = first
        // token of the sequence).  The ranges cannot overlap (the next one starts at least ceil(len / QT) further)
        // and the line is num_tokens / QT + num_seqs long, so a batch of one long and many short prompts launches
        // about as many workgroups as it has tiles, not longest-prompt tiles times sequences.
        extern __shared__ int32_t s_cu[];             // [num_seqs + 1]
        for (int i = threadIdx.x; i <= a.num_seqs; i += kPfThreads) s_cu[i] = a.cu_seqlens_q[i];
        __syncthreads();
        seq = 0;
        int hi = a.num_seqs;
        const int slot = (int)gridDim.y / a.kv_split - 1 - by;
        while (hi - seq > 1) { const int mid = (seq + hi) >> 1; if (s_cu[mid] / QT + mid <= slot) seq = mid; else hi = mid; }
        t0 = s_cu[seq];
        q_len = s_cu[seq + 1] - t0;
        qt = slot - (t0 / QT + seq);
        if (qt * QT >= q_len) return;
    } else {
        seq = blockIdx.y;
        t0 = a.cu_seqlens_q[seq];
        q_len = a.cu_seqlens_q[seq + 1] - t0;
        qt = (q_len + QT - 1) / QT - 1 - by;
        if (qt < 0) return;
    }
    if (a.skip_single && q_len == 1) return;
    const int ctx = a.ctx_lens[seq];
    const int n_keys = ctx + q_len;
    const int hk = h / (a.n_q_heads / a.n_kv_heads);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int col = lane & 15, c = lane >> 4;

    const int j0 = qt * QT + wave * QW;                        // first query row of this wave
    int jq[QB], q_pos[QB];                                     // this lane's query column in each column block
#pragma unroll
    for (int b = 0; b < QB; ++b) { jq[b] = j0 + 16 * b + col; q_pos[b] = ctx + jq[b]; }
    const int wave_last_pos = ctx + min(j0 + QW - 1, q_len - 1);
    const int wg_last_pos = ctx + min(qt * QT + QT - 1, q_len - 1);
    const int n_tiles = wg_last_pos / kPfKvTile + 1;
    const int n_pieces = kv_pieces(n_tiles, a.kv_split);
    if (piece >= n_pieces) return;
    const int tile_begin = (int)((int64_t)piece * n_tiles / n_pieces), tile_end = (int)((int64_t)(piece + 1) * n_tiles / n_pieces);

    // Q as column operand: lane holds Q[jq][32*ks + 8*c .. +7]
    u32x4 qreg[QB][KS];
#pragma unroll
    for (int b = 0; b < QB; ++b) {
        const uint16_t *qp = a.q + ((int64_t)(t0 + min(jq[b], q_len - 1)) * a.n_q_heads + h) * D + c * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qreg[b][ks] = ld16(qp + ks * 32);
    }
    f32x4_t o[QB][DT];
    float m_run[QB], l_run[QB];
#pragma unroll
    for (int b = 0; b < QB; ++b) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) o[b][dt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        m_run[b] = -INFINITY;
        l_run[b] = 0.f;
    }

    const int64_t head_elems = (int64_t)kBlockTokens * D;
    const int64_t unit_elems = 2 * (int64_t)a.n_kv_heads * head_elems;
    const uint16_t *layer_base = a.pool + (int64_t)a.layer_local * a.num_blocks * unit_elems;
    const int32_t *table = a.block_table + (int64_t)seq * a.max_blocks_per_seq;
    constexpr int kChunksPerRow = D / 8;
    constexpr int kChunksPerThread = kPfKvTile * kChunksPerRow / kPfThreads;

    // The K and V rows of the next tile travel from the cache to registers while the current tile is being multiplied.
    // Nothing between the request and the LDS store of the following iteration may need the loaded values (the memory
    // counter is in order: one early use would wait for everything requested before it), so rows past the sequence end
    // are dealt with at the store (V, last tile only: a zero probability must not meet an uninitialised NaN; a K row
    // past the end only produces scores that the causal mask replaces), and the block-table entries are not looked up
    // per tile: each lane keeps one entry of a 64-block (16-tile) stretch of the table, the next stretch is requested
    // sixteen tiles before it is needed, and a tile's entries are read out of those registers by lane index.
    // Thread tid owns chunk dc0 of rows r0 + i * kRowsPerPass of a tile; kRowsPerPass is a multiple of the cache
    // block, so its slot inside a block and its byte offset inside a unit never change, and the block a row lies in
    // is the same for all lanes of a wavefront.
    constexpr int kRowsPerPass = kPfThreads / kChunksPerRow;
    constexpr int kBlocksPerPass = kRowsPerPass / kBlockTokens, kBlocksPerTile = kPfKvTile / kBlockTokens;
    constexpr int kTilesPerStretch = 64 / kBlocksPerTile;
    static_assert(kRowsPerPass % kBlockTokens == 0, "a pass of the staging loop covers whole cache blocks");
    static_assert((64 / kChunksPerRow) <= kBlockTokens && kBlockTokens % (64 / kChunksPerRow) == 0, "the rows of a wavefront lie in one cache block");
    const int r0 = tid / kChunksPerRow, dc0 = tid % kChunksPerRow;
    const int wave_blk = __builtin_amdgcn_readfirstlane(r0 / kBlockTokens);      // block (within a pass) of this wavefront's rows
    const uint16_t *lane_base = layer_base + (int64_t)hk * head_elems + (int64_t)(r0 % kBlockTokens) * D + dc0 * 8;
    const int64_t v_off = (int64_t)a.n_kv_heads * head_elems;
    const int last_blk = (n_keys - 1) / kBlockTokens;
    const int last_tile = (n_keys - 1) / kPfKvTile;
    int32_t stretch_cur = table[min(tile_begin * kBlocksPerTile + lane, last_blk)];
    int32_t stretch_next = table[min((tile_begin + kTilesPerStretch) * kBlocksPerTile + lane, last_blk)];
    u32x4 kreg[kChunksPerThread], vreg[kChunksPerThread];
    auto fetch_tile = [&](int tile) {
        const int in_stretch = (tile - tile_begin) % kTilesPerStretch;
        if (in_stretch == 0 && tile != tile_begin) {
            stretch_cur = stretch_next;
            stretch_next = table[min((tile + kTilesPerStretch) * kBlocksPerTile + lane, last_blk)];
        }
#pragma unroll
        for (int i = 0; i < kChunksPerThread; ++i) {
            const int32_t phys = __builtin_amdgcn_readlane(stretch_cur, in_stretch * kBlocksPerTile + i * kBlocksPerPass + wave_blk);
            const uint16_t *kp = lane_base + (int64_t)phys * unit_elems;
            kreg[i] = ld16(kp);
            vreg[i] = ld16(kp + v_off);
        }
    };
    // stage K and V (both row-major, padded pitches) of the tile held in registers
    auto store_tile = [&](int tile) {
        if (tile == last_tile) {
#pragma unroll
            for (int i = 0; i < kChunksPerThread; ++i)
                if (tile * kPfKvTile + r0 + i * kRowsPerPass >= n_keys) vreg[i] = u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int i = 0; i < kChunksPerThread; ++i) {
            const int r = r0 + i * kRowsPerPass;
            *reinterpret_cast<u32x4 *>(s_k + r * kKPitch + dc0 * 16) = kreg[i];
            *reinterpret_cast<u32x4 *>(s_v + r * kVPitch + dc0 * 16) = vreg[i];
        }
    };
    fetch_tile(tile_begin);

    for (int tile = tile_begin; tile < tile_end; ++tile) {
        const int kv0 = tile * kPfKvTile;
        __syncthreads();
        store_tile(tile);
        __syncthreads();
        if (tile + 1 < tile_end) fetch_tile(tile + 1);
        __builtin_amdgcn_sched_barrier(0);          // the requests go out before the products, not after them
        if (kv0 > wave_last_pos) continue;          // whole tile is in this wave's future (wave-uniform)

        // ---- S^T = K . Q^T for the 4 sub-tiles of 16 keys; a K operand read from LDS serves every column block
        // (below the diagonal every key of the tile is visible to every query row of the wave:
        // no mask arithmetic there)
        const bool full_tile = !DEBUG && kv0 + kPfKvTile - 1 <= ctx + j0;
        // The operands of the next sub-tile are requested before the products of the current one (the compiler
        // on its own asks for each operand right before its use and then waits out the LDS latency 8 times per phase);
        // the scheduling barriers keep that order.
        f32x4_t acc[QB][4];
        u32x4 kop[2][KS];
        auto read_k = [&](int st, u32x4 (&dst)[KS]) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                dst[ks] = *reinterpret_cast<const u32x4 *>(s_k + (st * 16 + col) * kKPitch + ks * 64 + c * 16);
        };
        read_k(0, kop[0]);
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            if (st + 1 < 4) read_k(st + 1, kop[(st + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int b = 0; b < QB; ++b) acc[b][st] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int b = 0; b < QB; ++b)
                    acc[b][st] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kop[st & 1][ks]),
                                                                         __builtin_bit_cast(bf16x8_t, qreg[b][ks]), acc[b][st], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        // the first V^T operands travel while the softmax runs
        u32x4 vop[2][2];
        auto read_v = [&](int dt, u32x4 (&dst)[2]) {
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                // row operand: dim 16*dt + col; k slots 8c..8c+3 = keys 32u+4c.., 8c+4.. = keys 32u+16+4c..
                // LDS transpose load: lane j' of a 16-lane group points at key 4c + j'/4, dims
                // 4*(j'%4)..+3 of the tile; the hardware hands lane i the four keys of dim i.
                const char *vsrc = s_v + (32 * u + 4 * c + (col >> 2)) * kVPitch + dt * 32 + (col & 3) * 8;
                const u32x2 lo = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s *)(vsrc)));
                const u32x2 hi = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s *)(vsrc + 16 * kVPitch)));
                dst[u] = u32x4{lo.x, lo.y, hi.x, hi.y};
            }
        };
        read_v(0, vop[0]);
        __builtin_amdgcn_sched_barrier(0);
        u32x4 pop[QB][2];                             // P^T column operands for sub-tile pairs (0,1) and (2,3)
#pragma unroll
        for (int b = 0; b < QB; ++b) {
            // scores stay unscaled: the scale (log2(e) / sqrt(D), positive) is applied inside the exponent's
            // multiply-add, and the running maximum is kept unscaled too
            float s[4][4];
            if (full_tile) {
#pragma unroll
                for (int st = 0; st < 4; ++st)
#pragma unroll
                    for (int v = 0; v < 4; ++v) s[st][v] = acc[b][st][v];
            } else {
#pragma unroll
                for (int st = 0; st < 4; ++st)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int kv = kv0 + st * 16 + 4 * c + v;
                        s[st][v] = (kv <= q_pos[b]) ? acc[b][st][v] : -INFINITY;
                        if constexpr (DEBUG) {
                            if (jq[b] < q_len && kv <= q_pos[b])
                                a.dbg_scores[((int64_t)(t0 + jq[b]) * a.n_q_heads + h) * a.dbg_stride + kv] = acc[b][st][v] * a.scale_log2e;
                        }
                    }
            }
            // ---- online softmax per query column (lanes col, col+16, col+32, col+48)
            float mx = m_run[b];
#pragma unroll
            for (int st = 0; st < 4; ++st)
#pragma unroll
                for (int v = 0; v < 4; ++v) mx = fmaxf(mx, s[st][v]);
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float ms = (mx == -INFINITY) ? 0.f : mx;
            const float alpha = __builtin_amdgcn_exp2f((m_run[b] - ms) * a.scale_log2e);
            m_run[b] = mx;
            const float neg_ms = -ms * a.scale_log2e;
            float psum = 0.f;
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                float p[8];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    p[v] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[2 * u][v], a.scale_log2e, neg_ms));
                    p[4 + v] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[2 * u + 1][v], a.scale_log2e, neg_ms));
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) psum += p[e];
                pop[b][u] = u32x4{pack_bf16x2(p[0], p[1]), pack_bf16x2(p[2], p[3]), pack_bf16x2(p[4], p[5]), pack_bf16x2(p[6], p[7])};
            }
            l_run[b] = l_run[b] * alpha + psum;       // per lane; the four lanes of a column are added once at the end
            // the accumulator rescale only when some row's maximum moved
            if (__builtin_amdgcn_ballot_w64(alpha != 1.f)) {
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) o[b][dt] *= alpha;
            }
        }
        // ---- O^T += V^T . P^T; a V^T operand read from LDS serves every column block
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            if (dt + 1 < DT) read_v(dt + 1, vop[(dt + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int b = 0; b < QB; ++b)
                    o[b][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, vop[dt & 1][u]),
                                                                       __builtin_bit_cast(bf16x8_t, pop[b][u]), o[b][dt], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

#pragma unroll
    for (int b = 0; b < QB; ++b) {
        float l = l_run[b];
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        if (jq[b] >= q_len) continue;
        if (n_pieces > 1) {
            // one piece of several: unnormalised sums, running maximum and denominator go to the merge kernel.  A wave whose
            // rows see none of this piece's keys hands over m = -inf, l = 0, o = 0.
            const int64_t row = ((int64_t)piece * a.num_tokens + t0 + jq[b]) * a.n_q_heads + h;
            float *pa = a.part_acc + row * D + 4 * c;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) *reinterpret_cast<f32x4_t *>(pa + dt * 16) = o[b][dt];
            if (c == 0) { a.part_ml[row * 2] = m_run[b] * a.scale_log2e; a.part_ml[row * 2 + 1] = l; }
            continue;
        }
        const float inv = 1.f / l;
        uint16_t *op = a.out + ((int64_t)(t0 + jq[b]) * a.n_q_heads + h) * D + 4 * c;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            const u32x2 w = {pack_bf16x2(o[b][dt][0] * inv, o[b][dt][1] * inv), pack_bf16x2(o[b][dt][2] * inv, o[b][dt][3] * inv)};
            *reinterpret_cast<u32x2 *>(op + dt * 16) = w;
        }
        if constexpr (DEBUG) {
            if (c == 0) {
                float *ml = a.dbg_ml + ((int64_t)(t0 + jq[b]) * a.n_q_heads + h) * 3;
                ml[0] = m_run[b] * a.scale_log2e; ml[1] = l; ml[2] = __int_as_float(q_pos[b] + 1);
            }
        }
    }
}

// Merge of the pieces of the query tiles whose keys were cut: out = sum_z 2^(m_z - M) o_z / sum_z 2^(m_z - M) l_z.
// One thread per four output dims; rows whose tile ran as one piece were finished by the attention kernel.
template <int D>
__global__ __launch_bounds__(kPfThreads) void attn_prefill_merge_kernel(PrefillAttnArgs a)
{
    constexpr int kLanesPerRow = D / 4, kRowsPerWg = kPfThreads / kLanesPerRow;
    const int64_t row = (int64_t)blockIdx.x * kRowsPerWg + threadIdx.x / kLanesPerRow;
    if (row >= (int64_t)a.num_tokens * a.n_q_heads) return;
    const int t = (int)(row / a.n_q_heads), i = threadIdx.x % kLanesPerRow;
    const int seq = a.tok_seq[t];
    const int t0 = a.cu_seqlens_q[seq], q_len = a.cu_seqlens_q[seq + 1] - t0;
    if (a.skip_single && q_len == 1) return;
    const int qt = (t - t0) / a.q_tile;
    const int wg_last_pos = a.ctx_lens[seq] + min(qt * a.q_tile + a.q_tile - 1, q_len - 1);
    const int n_pieces = kv_pieces(wg_last_pos / kPfKvTile + 1, a.kv_split);
    if (n_pieces == 1) return;
    const int64_t piece_stride = (int64_t)a.num_tokens * a.n_q_heads;
    float m = -INFINITY;
    for (int z = 0; z < n_pieces; ++z) m = fmaxf(m, a.part_ml[(row + z * piece_stride) * 2]);
    f32x4_t num = {0.f, 0.f, 0.f, 0.f};
    float den = 0.f;
    for (int z = 0; z < n_pieces; ++z) {
        const int64_t r = row + z * piece_stride;
        const float wgt = __builtin_amdgcn_exp2f(a.part_ml[r * 2] - m);     // piece 0 always holds key 0, so m is finite
        den += wgt * a.part_ml[r * 2 + 1];
        num += wgt * *reinterpret_cast<const f32x4_t *>(a.part_acc + r * D + 4 * i);
    }
    const float inv = 1.f / den;
    const u32x2 w = {pack_bf16x2(num[0] * inv, num[1] * inv), pack_bf16x2(num[2] * inv, num[3] * inv)};
    *reinterpret_cast<u32x2 *>(a.out + row * D + 4 * i) = w;
}

// debug only: scores (log2 domain) -> probabilities, one workgroup per (token, head)
__global__ void attn_probs_normalize_kernel(float *scores, const float *ml, int64_t stride)
{
    const int64_t row = blockIdx.x;
    const float m = ml[row * 3], l = ml[row * 3 + 1];
    const int n = __float_as_int(ml[row * 3 + 2]);
    for (int r = threadIdx.x; r < n; r += blockDim.x)
        scores[row * stride + r] = __builtin_amdgcn_exp2f(scores[row * stride + r] - m) / l;
}

// Query rows per workgroup: 128 (two column blocks per wave) or 64.  The wide tile has the higher throughput and the
// longer critical path (the last tile of a prompt walks all its keys at twice the work per step), so it needs enough
// tiles to keep the chip busy past the long ones -- measured with 32 heads: one prompt of 2048 tokens (512 wide tiles)
// is 10 % faster on 64-row tiles, one of 3072 (768) 16 % faster on 128-row tiles, several prompts break even at 512 --
// or, with fewer, a block table with room for a cached prefix of at least two key pieces besides the longest chunk
// (then the walks are long and even, and cut keys fill the chip: 512 tokens behind 8192 cached: 146 -> 122 us).
int prefill_q_tile(int n_q_heads, int num_tokens, int num_seqs, int max_q_len, int max_blocks_per_seq)
{
    static const int forced = tuning_int("FXP_PREFILL_Q_TILE", 0);
    if (forced == 64 || forced == 128) return forced;
    if (num_tokens < 128 * (int64_t)std::max(num_seqs, 1)) return 64;
    const int64_t tiles = (int64_t)n_q_heads * (num_tokens / 128);
    if (tiles >= prefill_resident_wgs(64)) return 128;
    const bool prefix_room = (int64_t)max_blocks_per_seq * kBlockTokens - max_q_len >= 2 * kPfMinPieceTiles * kPfKvTile;
    return prefix_room && tiles * kPfMaxPieces >= prefill_resident_wgs(128) ? 128 : 64;
}
size_t prefill_piece_rows(int n_q_heads, int max_tokens)
{
    // rows of [piece][token][head]: pieces * heads * tiles <= the resident workgroups, q_tile tokens per tile, pieces <= kPfMaxPieces
    const size_t by_wgs = std::max((size_t)prefill_resident_wgs(64) * 64, (size_t)prefill_resident_wgs(128) * 128);
    return std::min<size_t>(by_wgs, (size_t)kPfMaxPieces * (size_t)std::max(max_tokens, 1) * n_q_heads);
}
int prefill_kv_split(int n_q_heads, int num_tokens, int num_seqs, int max_blocks_per_seq, int q_tile)
{
    static const int forced = tuning_int("FXP_PREFILL_KV_SPLIT", 0);
    const int64_t rows = (int64_t)std::max(num_tokens, 1) * n_q_heads;
    const int64_t fits = (int64_t)prefill_piece_rows(n_q_heads, num_tokens) / rows;      // pieces the workspace has rows for
    if (forced > 0) return (int)std::max<int64_t>(1, std::min<int64_t>(std::min(forced, kPfMaxPieces), fits));
    // no sequence can hold two pieces' worth of keys: nothing to cut
    if ((int64_t)max_blocks_per_seq * kBlockTokens < 2 * kPfMinPieceTiles * kPfKvTile) return 1;
    const int64_t wgs = (int64_t)n_q_heads * (num_tokens / q_tile + num_seqs);      // upper bound of the live workgroups
    return (int)std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(kPfMaxPieces, prefill_resident_wgs(q_tile) / wgs), fits));
}

template <int D, int QB>
static hipError_t launch_q(const PrefillAttnArgs &a_in, hipStream_t stream)
{
    constexpr int QT = 64 * QB;
    PrefillAttnArgs a = a_in;
    // the tile index and the piece share one grid dimension of at most 65535 (both kernels read the factor from here)
    const int64_t widest = std::max<int64_t>((a.max_q_len + QT - 1) / QT, a.num_tokens / QT + a.num_seqs);
    while (a.kv_split > 1 && widest * a.kv_split > 65535) --a.kv_split;
    if (widest > 65535 || a.num_seqs > 65535) return hipErrorInvalidValue;
    // one line of tiles when the rectangle (tiles of the longest prompt x sequences) would be more than eight times as
    // large (an empty workgroup costs a few nanoseconds, which only matters when there are very many of them)
    const int rect_x = (a.max_q_len + QT - 1) / QT, flat_x = a.num_tokens / QT + a.num_seqs;
    static const int forced = tuning_int("FXP_PREFILL_FLAT_GRID", -1);
    const bool flat = forced >= 0 ? forced != 0 : (int64_t)rect_x * a.num_seqs > 8 * (int64_t)flat_x;
    const dim3 grid = flat ? dim3(a.n_q_heads, flat_x * a.kv_split) : dim3(a.n_q_heads, a.num_seqs, rect_x * a.kv_split);
    const size_t lds = flat ? (size_t)(a.num_seqs + 1) * sizeof(int32_t) : 0;
    if constexpr (QB == 1) {
        if (a.dbg_scores) {
            if (flat) hipLaunchKernelGGL((attn_prefill_kernel<D, 1, true, true>), grid, dim3(kPfThreads), lds, stream, a);
            else hipLaunchKernelGGL((attn_prefill_kernel<D, 1, true, false>), grid, dim3(kPfThreads), lds, stream, a);
            hipLaunchKernelGGL(attn_probs_normalize_kernel, dim3(a.num_tokens * a.n_q_heads), dim3(64), 0, stream,
                               a.dbg_scores, a.dbg_ml, a.dbg_stride);
            return hipGetLastError();
        }
    }
    if (flat) hipLaunchKernelGGL((attn_prefill_kernel<D, QB, false, true>), grid, dim3(kPfThreads), lds, stream, a);
    else hipLaunchKernelGGL((attn_prefill_kernel<D, QB, false, false>), grid, dim3(kPfThreads), lds, stream, a);
    if (a.kv_split > 1) {
        constexpr int kRowsPerWg = kPfThreads / (D / 4);
        const int64_t rows = (int64_t)a.num_tokens * a.n_q_heads;
        hipLaunchKernelGGL((attn_prefill_merge_kernel<D>), dim3((unsigned)((rows + kRowsPerWg - 1) / kRowsPerWg)), dim3(kPfThreads), 0, stream, a);
    }
    return hipGetLastError();
}

template <int D>
static hipError_t launch_d(const PrefillAttnArgs &a_in, hipStream_t stream)
{
    PrefillAttnArgs a = a_in;
    // the probability dump runs every tile as one piece, 64 rows per workgroup
    if (a.dbg_scores || !a.part_acc || a.kv_split < 1) a.kv_split = 1;
    if (a.dbg_scores || a.q_tile != 128) a.q_tile = 64;
    return a.q_tile == 128 ? launch_q<D, 2>(a, stream) : launch_q<D, 1>(a, stream);
}

hipError_t launch_attn_prefill(const PrefillAttnArgs &a, hipStream_t stream)
{
    if (a.head_dim == 128) return launch_d<128>(a, stream);
    if (a.head_dim == 64) return launch_d<64>(a, stream);
    return hipErrorInvalidValue;
}

}  // namespace fxp
