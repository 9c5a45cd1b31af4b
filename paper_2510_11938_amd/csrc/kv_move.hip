// KV block mover: fused repartition (pool -> pool through both block tables),
// pack (pool -> contiguous buffer) and unpack (contiguous buffer -> pool).
//
// What is moved is fixed by the consistency rule of Section 6.3 (Eq. 10): the
// cache that arrives is the source cache multiplied element-wise by the token
// validity mask, so valid tokens arrive bit-identical and the invalid tail
// slots of a sequence's last block arrive as zero.
//
// An incremental pass moves only the tokens [from_i, to_i) of every sequence (the
// transfer runs while decoding continues, so a snapshot pass is followed by
// delta passes): slots before from_i are left alone, slots from to_i on in the
// last block are zero.  The token-dense buffer carries exactly those rows,
// [sequence][layer][K,V][head][token - from_i][dim], without block padding.
//
// HBM-bound bit copy.  One launch moves every (job, layer, sequence, logical
// block) unit.  The lengths live on the device, so each workgroup derives the
// per-sequence block prefix sums itself (LDS scan over ctx_lens) and then walks
// a grid-strided list of equal-sized 32 KiB work items: no empty workgroups for
// short sequences, no host synchronisation, no scratch memory.  Every lane
// moves 16-byte vectors, eight loads in flight before the first store.
#include "kernels.h"
#include "common.hip.h"

namespace fxp {

constexpr int kMoveThreads = 256;
constexpr int kMoveVecPerThread = 8;                                    // 16-byte vectors in flight per lane
constexpr int kMoveChunkBytes = kMoveThreads * 16 * kMoveVecPerThread;  // 32 KiB per work item

int kv_move_chunk_bytes() { return kMoveChunkBytes; }

// Address of one (layer, sequence, logical block) unit on a pool or block-packed side.
// j_rel counts from the first block of the sequence's token range.
__device__ __forceinline__ const char *side_unit_ptr(const KvMoveSide &s, int layer, int seq, int j, int j_rel,
                                                     int blocks_before, int nblk_seq, int64_t unit_bytes)
{
    int64_t unit;
    if (s.table) {
        int32_t phys = s.table[(int64_t)seq * s.max_blocks_per_seq + j];
        unit = (int64_t)(layer - s.layer_base) * s.num_blocks + phys;
    } else {   // packed: [sequence][layer - layer_base][logical block]
        unit = (int64_t)blocks_before * s.n_layers + (int64_t)(layer - s.layer_base) * nblk_seq + j_rel;
    }
    return s.base + unit * unit_bytes;
}

// Exclusive scans over the sequences of (blocks, tokens) in the range [from_i, to_i) -> LDS.
// Each thread sums a contiguous run of sequences, then a log-step scan over the threads.
__device__ __forceinline__ void scan_ranges(const KvMoveArgs &a, int32_t *pre_blk, int32_t *pre_tok, int32_t (*part)[kMoveThreads])
{
    const int tid = threadIdx.x, n = a.num_seqs;
    const int per = (n + kMoveThreads - 1) / kMoveThreads;
    const int lo = min(tid * per, n), hi = min(lo + per, n);
    auto counts = [&](int i, int32_t &nb, int32_t &ntok) {
        const int32_t to = a.to_lens[i], from = a.from_lens ? a.from_lens[i] : 0;
        const bool ok = from >= 0 && to > from;                       // empty or malformed range: nothing moves
        nb = ok ? (to + kBlockTokens - 1) / kBlockTokens - from / kBlockTokens : 0;
        ntok = ok ? to - from : 0;
    };
    int32_t lb = 0, lt = 0;
    for (int i = lo; i < hi; ++i) { int32_t nb, ntok; counts(i, nb, ntok); lb += nb; lt += ntok; }
    part[0][tid] = lb; part[1][tid] = lt;
    __syncthreads();
    for (int o = 1; o < kMoveThreads; o <<= 1) {
        const int32_t vb = tid >= o ? part[0][tid - o] : 0, vt = tid >= o ? part[1][tid - o] : 0;
        __syncthreads();
        part[0][tid] += vb; part[1][tid] += vt;
        __syncthreads();
    }
    int32_t rb = part[0][tid] - lb, rt = part[1][tid] - lt;
    for (int i = lo; i < hi; ++i) { int32_t nb, ntok; counts(i, nb, ntok); pre_blk[i] = rb; pre_tok[i] = rt; rb += nb; rt += ntok; }
    if (tid == kMoveThreads - 1) { pre_blk[n] = part[0][tid]; pre_tok[n] = part[1][tid]; }
    __syncthreads();
}

// TOKEN_DENSE: one side of every job is a token-dense buffer
// [sequence][layer][K,V][head][token - from][dim]; its addresses are per token row.
// (the block-granular variant must fit 64 registers: the persistent grid is sized for 8 workgroups
// per CU and all of them have to be resident)
template <bool TOKEN_DENSE>
__global__ __launch_bounds__(kMoveThreads, TOKEN_DENSE ? 4 : 8) void kv_move_kernel(KvMoveArgs a)
{
    extern __shared__ int32_t s_dyn[];         // [num_seqs + 1] blocks, [num_seqs + 1] tokens before each sequence
    __shared__ int32_t part[2][kMoveThreads];
    const int tid = threadIdx.x;
    const int n = a.num_seqs;
    int32_t *prefix = s_dyn, *pre_tok = s_dyn + n + 1;
    scan_ranges(a, prefix, pre_tok, part);
    const int64_t total_blocks = prefix[n];
    if (total_blocks == 0) return;

    const int64_t unit_bytes = a.unit_bytes;
    const int chunks = (int)((unit_bytes + kMoveChunkBytes - 1) / kMoveChunkBytes);
    const int row_bytes = a.head_dim * 2;                 // one token row of one head
    const int head_bytes = row_bytes * kBlockTokens;      // one (K or V, head) of a block
    const int rows_per_unit = (int)(unit_bytes / head_bytes);   // 2 * Hkv
    int64_t total_items = 0;
    for (int jb = 0; jb < a.n_jobs; ++jb)
        total_items += total_blocks * (a.jobs[jb].layer_end - a.jobs[jb].layer_begin) * chunks;

    for (int64_t item = blockIdx.x; item < total_items; item += gridDim.x) {
        int jb = 0;
        int64_t r = item;
        for (;; ++jb) {      // job that owns this item (jobs are few)
            const int64_t cnt = total_blocks * (a.jobs[jb].layer_end - a.jobs[jb].layer_begin) * chunks;
            if (r < cnt) break;
            r -= cnt;
        }
        const KvMoveJob &job = a.jobs[jb];
        const int chunk = (int)(r % chunks); r /= chunks;
        const int b = (int)(r % total_blocks);
        const int layer = job.layer_begin + (int)(r / total_blocks);
        // sequence that owns global block index b: prefix[seq] <= b < prefix[seq+1]
        int s_lo = 0, s_hi = n;
        while (s_hi - s_lo > 1) { int mid = (s_lo + s_hi) >> 1; if (prefix[mid] <= b) s_lo = mid; else s_hi = mid; }
        const int seq = s_lo;
        const int before = prefix[seq];
        const int nblk_seq = prefix[seq + 1] - before;
        const int32_t from = a.from_lens ? a.from_lens[seq] : 0, to = a.to_lens[seq];
        const int j_rel = b - before, j = from / kBlockTokens + j_rel;      // logical block of the sequence
        const int lo_slot = max(0, from - j * kBlockTokens);                 // slots below belong to an earlier pass
        const int hi_slot = min(kBlockTokens, to - j * kBlockTokens);        // slots from here on are masked out

        const char *sp = nullptr;
        char *dp = nullptr;
        if (!TOKEN_DENSE || job.src.token_dense == 0) sp = side_unit_ptr(job.src, layer, seq, j, j_rel, before, nblk_seq, unit_bytes);
        if (!TOKEN_DENSE || job.dst.token_dense == 0) dp = const_cast<char *>(side_unit_ptr(job.dst, layer, seq, j, j_rel, before, nblk_seq, unit_bytes));
        if (!TOKEN_DENSE) {
            if (job.dst.limit_bytes && (dp - job.dst.base) + unit_bytes > job.dst.limit_bytes) continue;   // never past a packed buffer
            if (job.src.limit_bytes && (sp - job.src.base) + unit_bytes > job.src.limit_bytes) continue;
        }
        // token-dense side: row of (layer, K|V head kvh, token t) =
        //   tokens_before * layers * 2Hkv + ((layer - layer_base) * 2Hkv + kvh) * ntok + (t - from)
        const KvMoveSide &dense = job.src.token_dense ? job.src : job.dst;
        const int64_t ntok = to - from;
        const int64_t dense_row0 = TOKEN_DENSE ? (int64_t)pre_tok[seq] * dense.n_layers * rows_per_unit
                                                 + (int64_t)(layer - dense.layer_base) * rows_per_unit * ntok
                                                 + (int64_t)j * kBlockTokens - from : 0;

        // offsets inside a unit fit 32 bits (a unit is 64 * Hkv * D bytes); slot index by 32-bit arithmetic
        const uint32_t ub = (uint32_t)unit_bytes, rb = (uint32_t)row_bytes;
        const uint32_t off0 = (uint32_t)chunk * kMoveChunkBytes + (uint32_t)tid * 16;
        u32x4 v[kMoveVecPerThread];
        int64_t dense_off[kMoveVecPerThread];
#pragma unroll
        for (int u = 0; u < kMoveVecPerThread; ++u) {
            const uint32_t off = off0 + (uint32_t)u * kMoveThreads * 16;
            const uint32_t row = off / rb;
            const int slot = (int)(row % kBlockTokens);
            bool move = off < ub && slot >= lo_slot && slot < hi_slot;
            if (TOKEN_DENSE) {
                const int kvh = (int)(row / kBlockTokens);
                dense_off[u] = (dense_row0 + (int64_t)kvh * ntok + slot) * row_bytes + (off - row * rb);
                if (dense.limit_bytes && dense_off[u] + 16 > dense.limit_bytes) move = false;             // never past the buffer
            }
            v[u] = u32x4{0u, 0u, 0u, 0u};
            if (move) {
                const char *p = (TOKEN_DENSE && job.src.token_dense) ? job.src.base + dense_off[u] : sp + off;
                v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
            }
        }
#pragma unroll
        for (int u = 0; u < kMoveVecPerThread; ++u) {
            const uint32_t off = off0 + (uint32_t)u * kMoveThreads * 16;
            const int slot = (int)((off / rb) % kBlockTokens);
            if (off >= ub || slot < lo_slot) continue;
            if (TOKEN_DENSE && job.dst.token_dense) {
                if (slot < hi_slot && !(dense.limit_bytes && dense_off[u] + 16 > dense.limit_bytes))
                    __builtin_nontemporal_store(v[u], reinterpret_cast<u32x4 *>(job.dst.base + dense_off[u]));
            } else {
                if (TOKEN_DENSE && slot < hi_slot && dense.limit_bytes && dense_off[u] + 16 > dense.limit_bytes) continue;   // row was not in the buffer
                __builtin_nontemporal_store(v[u], reinterpret_cast<u32x4 *>(dp + off));                   // masked slots: zero
            }
        }
    }
}


hipError_t launch_kv_move(const KvMoveArgs &args, int grid, hipStream_t stream)
{
    size_t lds = 2 * (size_t)(args.num_seqs + 1) * sizeof(int32_t);
    bool dense = false;
    for (int j = 0; j < args.n_jobs; ++j) dense = dense || args.jobs[j].src.token_dense || args.jobs[j].dst.token_dense;
    if (dense) hipLaunchKernelGGL(kv_move_kernel<true>, dim3(grid), dim3(kMoveThreads), lds, stream, args);
    else hipLaunchKernelGGL(kv_move_kernel<false>, dim3(grid), dim3(kMoveThreads), lds, stream, args);
    return hipGetLastError();
}

}  // namespace fxp
