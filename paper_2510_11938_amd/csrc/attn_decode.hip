// Paged decode attention: one new query token per sequence against the
// sequence's cached keys and values, read through the block table.
//
// Bound by streaming the cache from HBM (every cached K and V byte is read
// exactly once per step, also with grouped query heads: the G query heads of a
// KV head are handled by the same lanes).  Contexts in a batch are ragged, so
// the work is not cut per sequence but as one line:
//   unit   = one 16-token cache block of one (sequence, kv head); all units of
//            the batch are numbered (sequence, kv head, block);
//   worker = one wavefront; worker w owns the units [w*U/W, (w+1)*U/W), so every
//            worker streams the same number of blocks (+-1) whatever the length
//            mix, and the whole grid starts and ends together.  The cut depends
//            on the lengths only, never on the physical placement of blocks;
//            (with head_group = Gs > 1 a worker is Gs neighbouring wavefronts of a
//            workgroup and a unit one block of Gs adjacent kv heads: the wavefronts
//            walk the same blocks at the same time, one head each, so the K runs
//            they ask for are one contiguous Gs*4 KiB stretch of the cache, which
//            HBM serves a few per cent faster than unrelated 4 KiB runs)
//   piece  = the part of one (sequence, kv head) inside a worker's range; the
//            worker leaves one partial softmax state (max, sum, acc[D]) per piece
//            and a second kernel merges the pieces of each head in worker order.
// Inside a worker a block's K (and V) for one head is one contiguous 16*D*2-byte
// run; a wave load instruction covers 1 KiB of it: D/8 lanes per token row, 16
// bytes (8 dims) per lane.  The q.k dot product is 8 FMAs per lane plus a
// log2(D/8)-step butterfly inside the row's lanes.  Each group of D/8 lanes keeps
// its own running (max, sum, acc[8]) over the token rows it sees, so the block
// loop has no other cross-lane traffic; the groups are merged once per piece in a
// fixed order.  Two register buffers hold the next block while the current one is
// consumed.  Everything after the bf16 loads is float; results are
// bit-reproducible.
#include "kernels.h"
#include "common.hip.h"
#include <math.h>
#include <stdlib.h>

namespace fxp {

constexpr int kDecWaves = 4;
constexpr int kDecThreads = kDecWaves * 64;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// merge running softmax state (m2,l2,acc2) into (m,l,acc); log2 domain
template <int NV>
__device__ __forceinline__ void merge_state(float &m, float &l, float (&acc)[NV], float m2, float l2, const float (&acc2)[NV])
{
    const float mn = fmaxf(m, m2);
    const float ms = (mn == -INFINITY) ? 0.f : mn;
    const float a1 = fast_exp2(m - ms), a2 = fast_exp2(m2 - ms);
    l = l * a1 + l2 * a2;
#pragma unroll
    for (int e = 0; e < NV; ++e) acc[e] = acc[e] * a1 + acc2[e] * a2;
    m = mn;
}

// Workers that share the U units: never more than units (no empty ranges).  With very few sequences
// every head would leave a piece per worker, and merging dozens of pieces costs more than the shorter
// streams save: then at most eight workers per (sequence, head group) on average, unless that leaves a
// worker more than 16 blocks (1 sequence of 1024 tokens: attention + merge 28 -> 21 us).
__device__ __forceinline__ int64_t worker_count(int64_t available, int64_t U, int64_t seq_groups)
{
    return min(min(available, U), max(8 * seq_groups, U / 16));
}
// first unit of worker w when U units are cut into W ranges
__device__ __forceinline__ int64_t worker_begin(int64_t w, int64_t U, int64_t W) { return w * U / W; }
// worker that owns unit u
__device__ __forceinline__ int64_t worker_of(int64_t u, int64_t U, int64_t W) { return ((u + 1) * W + U - 1) / U - 1; }

// Blocks (per head) before each sequence, prefix[0..n] with prefix[i] = sum_{j<i} ceil((ctx_j+1)/16):
// computed once per forward call (the lengths are the same for every layer), copied to LDS here.
__device__ __forceinline__ void fetch_prefix(const int32_t *blk_prefix, int n, int32_t *s_prefix)
{
    for (int i = threadIdx.x; i <= n; i += blockDim.x) s_prefix[i] = blk_prefix[i];
    __syncthreads();
}

constexpr int kDecTblChunk = 256;   // block-table entries a wavefront stages in LDS at a time (even)

template <int D, int G, bool DEBUG>
__global__ __launch_bounds__(kDecThreads) void attn_decode_kernel(DecodeAttnArgs a)
{
    constexpr int LPT = D / 8;               // lanes per token row
    constexpr int TPI = 64 / LPT;            // token rows per wave load instruction
    constexpr int IPB = kBlockTokens / TPI;  // load instructions per block (K or V)

    extern __shared__ int32_t s_prefix[];    // [num_seqs + 1] blocks (per head) before each sequence
    __shared__ int32_t s_tbl_all[kDecWaves][kDecTblChunk];
    fetch_prefix(a.blk_prefix, a.num_seqs, s_prefix);
    int32_t *s_tbl = s_tbl_all[threadIdx.x >> 6];

    const int lane = threadIdx.x & 63;
    const int Hkv = a.n_kv_heads, Gs = a.head_group, Hg = Hkv / Gs;
    const int64_t U = (int64_t)s_prefix[a.num_seqs] * Hg;
    const int64_t W = worker_count((int64_t)gridDim.x * kDecWaves / Gs, U, (int64_t)a.num_seqs * Hg);
    const int wave_id = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * kDecWaves + (threadIdx.x >> 6)));
    const int64_t wk = wave_id / Gs;                                 // worker: Gs neighbouring wavefronts, one head each
    const int hi_w = wave_id % Gs;
    if (wk >= W) return;
    int64_t u = worker_begin(wk, U, W);
    const int64_t u_end = worker_begin(wk + 1, U, W);
    if (u >= u_end) return;

    const int dc = lane % LPT, ti = lane / LPT;
    const int64_t head_bytes = (int64_t)kBlockTokens * D * 2;
    const int64_t unit_bytes = 2 * (int64_t)Hkv * head_bytes;
    const char *layer_base = reinterpret_cast<const char *>(a.pool) + (int64_t)a.layer_local * a.num_blocks * unit_bytes;

    // sequence that owns unit u: prefix[seq]*Hg <= u < prefix[seq+1]*Hg
    int seq;
    {
        int lo = 0, hi = a.num_seqs;
        while (hi - lo > 1) { const int mid = (lo + hi) >> 1; if ((int64_t)s_prefix[mid] * Hg <= u) lo = mid; else hi = mid; }
        seq = lo;
    }

    while (u < u_end) {
        while ((int64_t)s_prefix[seq + 1] * Hg <= u) ++seq;
        seq = __builtin_amdgcn_readfirstlane(seq);                       // wave-uniform: keep the piece's bookkeeping in scalar registers
        const int nb_seq = __builtin_amdgcn_readfirstlane(s_prefix[seq + 1] - s_prefix[seq]);
        const int64_t r = u - (int64_t)__builtin_amdgcn_readfirstlane(s_prefix[seq]) * Hg;
        const int hg = (int)(r / nb_seq), blk0 = (int)(r % nb_seq);
        const int hk = hg * Gs + hi_w;
        const int nblk = (int)min((int64_t)(nb_seq - blk0), u_end - u);  // blocks of this piece
        const int n_keys = a.ctx_lens[seq] + 1;                          // cached tokens + the one appended this step
        const int tok_row = a.cu_seqlens_q[seq];                         // the sequence's token row (= seq in a pure decode step)
        const int32_t *trow = a.block_table + (int64_t)seq * a.max_blocks_per_seq + blk0;

        // query, pre-scaled by log2(e)/sqrt(D) so that probabilities are exp2(s - m)
        float q[G][8];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const u32x4 v = ld16(a.q + ((int64_t)tok_row * a.n_q_heads + hk * G + g) * D + dc * 8);
            q[g][0] = bf16_lo(v.x) * a.scale_log2e; q[g][1] = bf16_hi(v.x) * a.scale_log2e;
            q[g][2] = bf16_lo(v.y) * a.scale_log2e; q[g][3] = bf16_hi(v.y) * a.scale_log2e;
            q[g][4] = bf16_lo(v.z) * a.scale_log2e; q[g][5] = bf16_hi(v.z) * a.scale_log2e;
            q[g][6] = bf16_lo(v.w) * a.scale_log2e; q[g][7] = bf16_hi(v.w) * a.scale_log2e;
        }
        float m[G], l[G], acc[G][8];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            m[g] = -INFINITY; l[g] = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;
        }

        // The table entries of the piece are staged in this wavefront's LDS region, a chunk at a
        // time.  A table load from global memory inside the block loop would make every wait for
        // it drain the (in-order) vector-memory counter, i.e. stall until the cache block in
        // flight has landed before the next one could be requested; LDS has a counter of its own.
        int c0 = 0;
        // K and V of a block are requested at different times (K before the scores of the previous
        // block, V after them): the two 4 KiB runs of one block lie exactly Hkv*4 KiB apart in the
        // same cache unit, and asking for both at once costs a few per cent of HBM bandwidth.
        auto block_ptr = [&](int b) {
            const int32_t phys = __builtin_amdgcn_readfirstlane(s_tbl[b - c0]);
            return layer_base + (int64_t)phys * unit_bytes + (int64_t)hk * head_bytes + lane * 16;
        };
        auto load_k = [&](int b, u32x4(&k)[IPB]) {
            const char *kp = block_ptr(b);
#pragma unroll
            for (int i = 0; i < IPB; ++i) k[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(kp + i * 1024));
        };
        auto load_v = [&](int b, u32x4(&v)[IPB]) {
            const char *vp = block_ptr(b) + (int64_t)Hkv * head_bytes;
#pragma unroll
            for (int i = 0; i < IPB; ++i) v[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(vp + i * 1024));
        };
        // scores of block b against the query, running maximum and sum; leaves the block's
        // probabilities p and the rescale factor alpha for weigh()
        float p[G][IPB], alpha[G];
        auto scores = [&](int b, const u32x4(&k)[IPB]) {
            const int tbase = (blk0 + b) * kBlockTokens;
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float s[IPB];
#pragma unroll
                for (int i = 0; i < IPB; ++i) {
                    float d = q[g][0] * bf16_lo(k[i].x);
                    d = fmaf(q[g][1], bf16_hi(k[i].x), d);
                    d = fmaf(q[g][2], bf16_lo(k[i].y), d);
                    d = fmaf(q[g][3], bf16_hi(k[i].y), d);
                    d = fmaf(q[g][4], bf16_lo(k[i].z), d);
                    d = fmaf(q[g][5], bf16_hi(k[i].z), d);
                    d = fmaf(q[g][6], bf16_lo(k[i].w), d);
                    d = fmaf(q[g][7], bf16_hi(k[i].w), d);
#pragma unroll
                    for (int o = LPT / 2; o > 0; o >>= 1) d += __shfl_xor(d, o, 64);
                    const int tok = tbase + i * TPI + ti;
                    s[i] = tok < n_keys ? d : -INFINITY;
                    if constexpr (DEBUG) {
                        if (dc == 0 && tok < n_keys)
                            a.dbg_scores[((int64_t)tok_row * a.n_q_heads + hk * G + g) * a.dbg_stride + tok] = d;
                    }
                }
                float mn = m[g];
#pragma unroll
                for (int i = 0; i < IPB; ++i) mn = fmaxf(mn, s[i]);
                const float ms = (mn == -INFINITY) ? 0.f : mn;
                alpha[g] = fast_exp2(m[g] - ms);
                m[g] = mn;
                float psum = 0.f;
#pragma unroll
                for (int i = 0; i < IPB; ++i) { p[g][i] = fast_exp2(s[i] - ms); psum += p[g][i]; }
                l[g] = l[g] * alpha[g] + psum;
            }
        };
        // acc = acc * alpha + p . V of block b
        auto weigh = [&](int b, u32x4(&v)[IPB]) {
            const int tbase = (blk0 + b) * kBlockTokens;
            if (tbase + kBlockTokens > n_keys) {
                // last block of the sequence: rows past the end may hold anything (also NaN
                // patterns); zero them so that a zero probability meets a zero value
#pragma unroll
                for (int i = 0; i < IPB; ++i)
                    if (tbase + i * TPI + ti >= n_keys) v[i] = u32x4{0u, 0u, 0u, 0u};
            }
#pragma unroll
            for (int g = 0; g < G; ++g) {
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[g][e] *= alpha[g];
#pragma unroll
                for (int i = 0; i < IPB; ++i) {
                    acc[g][0] = fmaf(p[g][i], bf16_lo(v[i].x), acc[g][0]);
                    acc[g][1] = fmaf(p[g][i], bf16_hi(v[i].x), acc[g][1]);
                    acc[g][2] = fmaf(p[g][i], bf16_lo(v[i].y), acc[g][2]);
                    acc[g][3] = fmaf(p[g][i], bf16_hi(v[i].y), acc[g][3]);
                    acc[g][4] = fmaf(p[g][i], bf16_lo(v[i].z), acc[g][4]);
                    acc[g][5] = fmaf(p[g][i], bf16_hi(v[i].z), acc[g][5]);
                    acc[g][6] = fmaf(p[g][i], bf16_lo(v[i].w), acc[g][6]);
                    acc[g][7] = fmaf(p[g][i], bf16_hi(v[i].w), acc[g][7]);
                }
            }
        };

        // Software pipeline over register buffers.  Loads inside the steady-state loop are
        // unconditional: a load under a branch makes the compiler wait for everything in
        // flight (also the block just requested) at the next use, which serialises the stream.
        for (c0 = 0; c0 < nblk; c0 += kDecTblChunk) {
            const int ce = min(c0 + kDecTblChunk, nblk);
            for (int j = lane; j < ce - c0; j += 64) s_tbl[j] = trow[c0 + j];
            __builtin_amdgcn_wave_barrier();
            int b = c0;
            // K runs two blocks ahead of the scores and is requested in the middle of an iteration, V
            // one block ahead and at its start: the K and the V request of one block are then most of
            // an iteration apart, with two register buffers each.
            u32x4 k0[IPB], v0[IPB], k1[IPB], v1[IPB];
            load_k(b, k0);
            if (b + 1 < ce) load_k(b + 1, k1);
            load_v(b, v0);
            while (b + 3 < ce) {
                load_v(b + 1, v1);
                scores(b, k0);
                load_k(b + 2, k0);
                weigh(b, v0);
                load_v(b + 2, v0);
                scores(b + 1, k1);
                load_k(b + 3, k1);
                weigh(b + 1, v1);
                b += 2;
            }
            // one to three blocks left: K(b), K(b+1) and V(b) have been requested
            if (b + 1 < ce) load_v(b + 1, v1);
            scores(b, k0);
            if (b + 2 < ce) load_k(b + 2, k0);
            weigh(b, v0);
            if (b + 1 < ce) {
                if (b + 2 < ce) load_v(b + 2, v0);
                scores(b + 1, k1);
                weigh(b + 1, v1);
                if (b + 2 < ce) { scores(b + 2, k0); weigh(b + 2, v0); }
            }
        }

        // merge the TPI lane groups (butterfly, lower group always the first operand) and store the piece
        // unique: consecutive pieces of a head differ in worker or in (sequence, head group), and never go back in either
        const int64_t slot = (wk + (int64_t)seq * Hg + hg) * Gs + hi_w;
#pragma unroll
        for (int g = 0; g < G; ++g) {
#pragma unroll
            for (int o = LPT; o < 64; o <<= 1) {
                float m2 = __shfl_xor(m[g], o, 64), l2 = __shfl_xor(l[g], o, 64), acc2[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) acc2[e] = __shfl_xor(acc[g][e], o, 64);
                if ((lane & o) == 0) merge_state<8>(m[g], l[g], acc[g], m2, l2, acc2);
                else {
                    float mm = m2, ll = l2;
                    merge_state<8>(mm, ll, acc2, m[g], l[g], acc[g]);
                    m[g] = mm; l[g] = ll;
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[g][e] = acc2[e];
                }
            }
            if (ti == 0) {
                float *pa = a.part_acc + (slot * G + g) * D + dc * 8;
                *reinterpret_cast<f32x4_t *>(pa) = f32x4_t{acc[g][0], acc[g][1], acc[g][2], acc[g][3]};
                *reinterpret_cast<f32x4_t *>(pa + 4) = f32x4_t{acc[g][4], acc[g][5], acc[g][6], acc[g][7]};
                if (dc == 0) { a.part_ml[(slot * G + g) * 2] = m[g]; a.part_ml[(slot * G + g) * 2 + 1] = l[g]; }
            }
        }
        u += nblk;
    }
}

// ---------------------------------------------------------------------------
// Grouped-query variant (2..16 query heads per kv head).  With G query heads the
// float pipe would need G FMAs per loaded K or V element and the kernel would be
// bound by vector ALU long before HBM, so both products run on the matrix cores,
// 32 keys (two cache blocks) at a time, with the same unit/worker/piece cut:
//   S^T[key][head]  = K[key][:] . Q[head][:]    row operand = K rows straight from
//                     the cache block, column operand = the group's query heads
//                     (columns >= G are zero);  the accumulator leaves lane
//                     (head j, group c) with keys 4c..4c+3 of each block;
//   softmax per head column: 8 in-lane values, two cross-lane steps for the max
//                     (the sum is kept per lane and reduced once per piece);
//   O^T[dim][head] += V^T[dim][key] . P^T[key][head]   P^T in accumulator layout
//                     is already the column operand (k slots 8c..8c+3 = block 0
//                     keys 4c.., 8c+4.. = block 1 keys 4c..); V^T is read with the
//                     LDS transpose load (ds_read_b64_tr_b16): the wave stores the
//                     two V blocks row-major in its own LDS region and lane
//                     (dim i, group c) receives V[key 4c+e][16*dt + i], e < 4.
// Probabilities enter the second product rounded to bf16.
template <int D, bool DEBUG>
__global__ __launch_bounds__(kDecThreads, 2) void attn_decode_mfma_kernel(DecodeAttnArgs a)
{
    constexpr int KS = D / 32;                 // k-steps of the score product
    constexpr int DT = D / 16;                 // 16-dim tiles of the output
    constexpr int kVPitch = D * 2 + 32;        // bytes per V row in LDS: 8 rows land in 8 distinct 32-byte bank groups
    constexpr int kVBlock = kBlockTokens * kVPitch;
    typedef short v4s __attribute__((ext_vector_type(4)));

    extern __shared__ int32_t s_dyn[];         // [num_seqs + 1] block prefix, then the per-wave V regions
    __shared__ int32_t s_tbl_all[kDecWaves][kDecTblChunk];
    int32_t *s_prefix = s_dyn;
    fetch_prefix(a.blk_prefix, a.num_seqs, s_prefix);
    int32_t *s_tbl = s_tbl_all[threadIdx.x >> 6];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 15, c = lane >> 4;
    const int Hkv = a.n_kv_heads, G = a.n_q_heads / Hkv;
    char *s_v = reinterpret_cast<char *>(s_dyn) + ((a.num_seqs + 1) * 4 + 255) / 256 * 256 + wave * (2 * kVBlock);
    const int Gs = a.head_group, Hg = Hkv / Gs;
    const int64_t U = (int64_t)s_prefix[a.num_seqs] * Hg;
    const int64_t W = worker_count((int64_t)gridDim.x * kDecWaves / Gs, U, (int64_t)a.num_seqs * Hg);
    const int wave_id = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * kDecWaves + wave));
    const int64_t wk = wave_id / Gs;                                 // worker: Gs neighbouring wavefronts, one kv head each
    const int hi_w = wave_id % Gs;
    if (wk >= W) return;
    int64_t u = worker_begin(wk, U, W);
    const int64_t u_end = worker_begin(wk + 1, U, W);
    if (u >= u_end) return;

    const int64_t head_bytes = (int64_t)kBlockTokens * D * 2;
    const int64_t unit_bytes = 2 * (int64_t)Hkv * head_bytes;
    const char *layer_base = reinterpret_cast<const char *>(a.pool) + (int64_t)a.layer_local * a.num_blocks * unit_bytes;

    int seq;
    {
        int lo = 0, hi = a.num_seqs;
        while (hi - lo > 1) { const int mid = (lo + hi) >> 1; if ((int64_t)s_prefix[mid] * Hg <= u) lo = mid; else hi = mid; }
        seq = lo;
    }
    // LDS addresses of this lane: where it stores V (row-major, 16 bytes per lane per load) and
    // where it points the transpose load (lane j' of a 16-lane group supplies key 4c + j'/4,
    // dims 4*(j'%4)..+3 of the 16-dim tile; the hardware hands lane i the four keys of dim i)
    const int v_tr = (4 * c + (col >> 2)) * kVPitch + (col & 3) * 8;               // + dt*32 + block*kVBlock

    while (u < u_end) {
        while ((int64_t)s_prefix[seq + 1] * Hg <= u) ++seq;
        seq = __builtin_amdgcn_readfirstlane(seq);
        const int nb_seq = __builtin_amdgcn_readfirstlane(s_prefix[seq + 1] - s_prefix[seq]);
        const int64_t r = u - (int64_t)__builtin_amdgcn_readfirstlane(s_prefix[seq]) * Hg;
        const int hg = (int)(r / nb_seq), blk0 = (int)(r % nb_seq);
        const int hk = hg * Gs + hi_w;
        const int nblk = (int)min((int64_t)(nb_seq - blk0), u_end - u);
        const int n_keys = a.ctx_lens[seq] + 1;
        const int tok_row = a.cu_seqlens_q[seq];
        const int32_t *trow = a.block_table + (int64_t)seq * a.max_blocks_per_seq + blk0;

        // column operand: query head col of the group (zero beyond G), dims 32*s + 8*c .. +7
        u32x4 qop[KS];
        {
            const uint16_t *qp = a.q + ((int64_t)tok_row * a.n_q_heads + hk * G + min(col, G - 1)) * D + c * 8;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const u32x4 v = ld16(qp + ks * 32);
                qop[ks] = col < G ? v : u32x4{0u, 0u, 0u, 0u};
            }
        }
        f32x4_t o[DT];
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) o[dt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        float m_run = -INFINITY, l_lane = 0.f;

        // loads of one pair of blocks (the second may be missing: it is then the first again, fully masked)
        int c0 = 0;
        auto load_pair = [&](int b, u32x4(&kop)[2][KS], u32x4(&vraw)[2][D / 32]) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int32_t phys = __builtin_amdgcn_readfirstlane(s_tbl[min(b + h, nblk - 1) - c0]);
                const char *kp = layer_base + (int64_t)phys * unit_bytes + (int64_t)hk * head_bytes;
                const char *vp = kp + (int64_t)Hkv * head_bytes;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)      // row operand: key col, dims 32*ks + 8*c
                    kop[h][ks] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(kp + col * (D * 2) + ks * 64 + c * 16));
#pragma unroll
                for (int i = 0; i < D / 32; ++i)     // plain row-major copy of the V block, 1 KiB per load
                    vraw[h][i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(vp + i * 1024 + lane * 16));
            }
        };
        auto consume_pair = [&](int b, const u32x4(&kop)[2][KS], const u32x4(&vraw)[2][D / 32]) {
            // V blocks -> this wave's LDS region (rows past the sequence end are zeroed: a zero
            // probability must not meet an uninitialised, possibly NaN, value)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int tbase = (blk0 + b + h) * kBlockTokens;
                const bool present = b + h < nblk;
#pragma unroll
                for (int i = 0; i < D / 32; ++i) {
                    constexpr int kRowsPerLoad = 1024 / (D * 2);     // 4 rows (D = 128) or 8 rows (D = 64) per load
                    const int row = i * kRowsPerLoad + (lane * 16) / (D * 2);
                    const bool ok = present && tbase + row < n_keys;
                    *reinterpret_cast<u32x4 *>(s_v + h * kVBlock + row * kVPitch + (lane * 16) % (D * 2)) =
                        ok ? vraw[h][i] : u32x4{0u, 0u, 0u, 0u};
                }
            }
            // scores of both blocks
            float sc[2][4];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kop[h][ks]),
                                                                  __builtin_bit_cast(bf16x8_t, qop[ks]), acc, 0, 0, 0);
                const int tbase = (blk0 + b + h) * kBlockTokens;
                const bool present = b + h < nblk;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int tok = tbase + 4 * c + v;
                    const float sv = acc[v] * a.scale_log2e;
                    const bool ok = present && tok < n_keys;
                    sc[h][v] = ok ? sv : -INFINITY;
                    if constexpr (DEBUG) {
                        if (ok && col < G) a.dbg_scores[((int64_t)tok_row * a.n_q_heads + hk * G + col) * a.dbg_stride + tok] = sv;
                    }
                }
            }
            float mx = m_run;
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int v = 0; v < 4; ++v) mx = fmaxf(mx, sc[h][v]);
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float ms = (mx == -INFINITY) ? 0.f : mx;
            const float alpha = fast_exp2(m_run - ms);
            m_run = mx;
            float p[8], psum = 0.f;
#pragma unroll
            for (int v = 0; v < 4; ++v) { p[v] = fast_exp2(sc[0][v] - ms); p[4 + v] = fast_exp2(sc[1][v] - ms); }
#pragma unroll
            for (int e = 0; e < 8; ++e) psum += p[e];
            l_lane = l_lane * alpha + psum;
            const u32x4 pop = {pack_bf16x2(p[0], p[1]), pack_bf16x2(p[2], p[3]), pack_bf16x2(p[4], p[5]), pack_bf16x2(p[6], p[7])};
            __builtin_amdgcn_wave_barrier();     // the V rows above are in LDS before the transpose loads below
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) v4s *)(s_v + v_tr + dt * 32));
                const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) v4s *)(s_v + kVBlock + v_tr + dt * 32));
                const u32x2 lo2 = __builtin_bit_cast(u32x2, lo), hi2 = __builtin_bit_cast(u32x2, hi);
                const u32x4 vop = {lo2.x, lo2.y, hi2.x, hi2.y};
                o[dt] *= alpha;
                o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, vop),
                                                                __builtin_bit_cast(bf16x8_t, pop), o[dt], 0, 0, 0);
            }
            __builtin_amdgcn_wave_barrier();     // the next pair's V stores stay behind these loads
        };

        // table entries through LDS and unconditional loads in the steady-state loop, as in the
        // kernel above
        for (c0 = 0; c0 < nblk; c0 += kDecTblChunk) {
            const int ce = min(c0 + kDecTblChunk, nblk);
            for (int j = lane; j < ce - c0; j += 64) s_tbl[j] = trow[c0 + j];
            __builtin_amdgcn_wave_barrier();
            u32x4 k0[2][KS], v0[2][D / 32], k1[2][KS], v1[2][D / 32];
            int b = c0;
            load_pair(b, k0, v0);
            while (b + 4 < ce) {
                load_pair(b + 2, k1, v1);
                consume_pair(b, k0, v0);
                load_pair(b + 4, k0, v0);
                consume_pair(b + 2, k1, v1);
                b += 4;
            }
            if (b + 2 < ce) load_pair(b + 2, k1, v1);
            consume_pair(b, k0, v0);
            if (b + 2 < ce) consume_pair(b + 2, k1, v1);
        }

        // the piece's state: sum over the four lane groups of a head column, then store
        float l_tot = l_lane;
        l_tot += __shfl_xor(l_tot, 16, 64);
        l_tot += __shfl_xor(l_tot, 32, 64);
        if (col < G) {
            const int64_t slot = (wk + (int64_t)seq * Hg + hg) * Gs + hi_w;
            float *pa = a.part_acc + (slot * G + col) * D + 4 * c;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) *reinterpret_cast<f32x4_t *>(pa + dt * 16) = o[dt];
            if (c == 0) { a.part_ml[(slot * G + col) * 2] = m_run; a.part_ml[(slot * G + col) * 2 + 1] = l_tot; }
        }
        u += nblk;
    }
}

// Merge the pieces of each (sequence, query head) in worker order and normalise:
// o = sum_p acc_p 2^(m_p - m) / sum_p l_p 2^(m_p - m).  One thread per dim of a (sequence, query head),
// 512 / D heads per workgroup.  The running maximum is carried along (as in the attention loop), so the
// maxima, sums and accumulators of a group of pieces are independent loads issued together: one
// memory round trip per four pieces instead of three dependent ones per piece.
template <bool DEBUG>
__global__ void attn_decode_combine_kernel(DecodeAttnArgs a)
{
    constexpr int kGroup = 4;
    const int D = a.head_dim, G = a.n_q_heads / a.n_kv_heads, Hkv = a.n_kv_heads;
    const int row_id = blockIdx.x * (blockDim.x / D) + threadIdx.x / D;      // (sequence, query head), several per workgroup
    if (row_id >= a.num_seqs * a.n_q_heads) return;
    const int seq = row_id / a.n_q_heads, head = row_id % a.n_q_heads, hk = head / G, g = head % G;
    const int tok_row = a.cu_seqlens_q[seq];
    if (a.cu_seqlens_q[seq + 1] - tok_row != 1) return;      // a prompt chunk in a mixed call: the prefill kernel's
    const int32_t before = a.blk_prefix[seq], total = a.blk_prefix[a.num_seqs];   // blocks (per head) before this sequence / in the batch
    const int n_keys = a.ctx_lens[seq] + 1;
    const int nb = (n_keys + kBlockTokens - 1) / kBlockTokens;
    const int Gs = a.head_group, Hg = Hkv / Gs, hg = hk / Gs, hi_w = hk % Gs;
    const int64_t U = (int64_t)total * Hg, W = worker_count((int64_t)a.n_workers / Gs, U, (int64_t)a.num_seqs * Hg);
    const int64_t u0 = (int64_t)before * Hg + (int64_t)hg * nb;
    const int64_t w_first = worker_of(u0, U, W), w_last = worker_of(u0 + nb - 1, U, W);
    const int64_t pair = (int64_t)seq * Hg + hg;
    const int d = threadIdx.x % D;
    float mm = -INFINITY, ll = 0.f, av = 0.f;
    for (int64_t w0 = w_first; w0 <= w_last; w0 += kGroup) {
        float m[kGroup], l[kGroup], ac[kGroup];
#pragma unroll
        for (int j = 0; j < kGroup; ++j) {
            const int64_t piece = ((min(w0 + j, w_last) + pair) * Gs + hi_w) * G + g;
            m[j] = a.part_ml[piece * 2];
            l[j] = a.part_ml[piece * 2 + 1];
            ac[j] = a.part_acc[piece * D + d];
        }
#pragma unroll
        for (int j = 0; j < kGroup; ++j) {
            if (w0 + j <= w_last) {
                const float mn = fmaxf(mm, m[j]);
                const float s_old = mm == -INFINITY ? 0.f : fast_exp2(mm - mn);
                const float s_new = m[j] == -INFINITY ? 0.f : fast_exp2(m[j] - mn);
                ll = ll * s_old + l[j] * s_new;
                av = av * s_old + ac[j] * s_new;
                mm = mn;
            }
        }
    }
    const int64_t row = (int64_t)tok_row * a.n_q_heads + head;
    a.out[row * D + d] = f32_to_bf16(av / ll);
    if constexpr (DEBUG) {
        // turn the stored scaled scores (log2 domain) into probabilities
        float *pr = a.dbg_scores + row * a.dbg_stride;
        for (int r = d; r < n_keys; r += D) pr[r] = fast_exp2(pr[r] - mm) / ll;
    }
}

template <int D, int G>
static hipError_t launch_dg(const DecodeAttnArgs &a, hipStream_t stream)
{
    const dim3 grid(a.n_workers / kDecWaves);
    const size_t lds = (size_t)(a.num_seqs + 1) * sizeof(int32_t);
    if (a.dbg_scores) hipLaunchKernelGGL((attn_decode_kernel<D, G, true>), grid, dim3(kDecThreads), lds, stream, a);
    else hipLaunchKernelGGL((attn_decode_kernel<D, G, false>), grid, dim3(kDecThreads), lds, stream, a);
    return hipGetLastError();
}

hipError_t launch_attn_decode_combine(const DecodeAttnArgs &a, hipStream_t stream)
{
    const int threads = 512, per_wg = threads / a.head_dim;      // query heads per workgroup: thousands of one-head workgroups take longer to launch than to run
    const dim3 cgrid((a.num_seqs * a.n_q_heads + per_wg - 1) / per_wg);
    if (a.dbg_scores) hipLaunchKernelGGL(attn_decode_combine_kernel<true>, cgrid, dim3(threads), 0, stream, a);
    else hipLaunchKernelGGL(attn_decode_combine_kernel<false>, cgrid, dim3(threads), 0, stream, a);
    return hipGetLastError();
}

int decode_head_group(int n_kv_heads)
{
    static const int forced = tuning_int("FXP_DECODE_HEAD_GROUP", 0);
    if (forced > 0 && kDecWaves % forced == 0 && n_kv_heads % forced == 0) return forced;
    return n_kv_heads % 4 == 0 ? 4 : (n_kv_heads % 2 == 0 ? 2 : 1);
}

bool decode_attn_supported(int head_dim, int group)
{
    return (head_dim == 64 || head_dim == 128) && group >= 1 && group <= 16;
}

template <int D>
static hipError_t launch_mfma(const DecodeAttnArgs &a, hipStream_t stream)
{
    const dim3 grid(a.n_workers / kDecWaves);
    const size_t lds = ((size_t)(a.num_seqs + 1) * 4 + 255) / 256 * 256 + (size_t)kDecWaves * 2 * kBlockTokens * (D * 2 + 32);
    if (a.dbg_scores) hipLaunchKernelGGL((attn_decode_mfma_kernel<D, true>), grid, dim3(kDecThreads), lds, stream, a);
    else hipLaunchKernelGGL((attn_decode_mfma_kernel<D, false>), grid, dim3(kDecThreads), lds, stream, a);
    return hipGetLastError();
}

hipError_t launch_attn_decode(const DecodeAttnArgs &a, hipStream_t stream)
{
    const int G = a.n_q_heads / a.n_kv_heads;
    if (G >= 2 && G <= 16) {          // grouped heads: matrix-core kernel
        if (a.head_dim == 128) return launch_mfma<128>(a, stream);
        if (a.head_dim == 64) return launch_mfma<64>(a, stream);
        return hipErrorInvalidValue;
    }
    if (a.head_dim == 128 && G == 1) return launch_dg<128, 1>(a, stream);
    if (a.head_dim == 64 && G == 1) return launch_dg<64, 1>(a, stream);
    return hipErrorInvalidValue;
}

}  // namespace fxp
