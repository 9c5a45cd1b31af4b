// KV block mover: fused repartition (pool -> pool through both block tables),
// pack (pool -> contiguous buffer) and unpack (contiguous buffer -> pool).
//
// What is moved is fixed by the consistency rule of Section 6.3 (Eq. 10): the
// cache that arrives is the source cache multiplied element-wise by the token
// validity mask, so valid tokens arrive bit-identical and the invalid tail
// slots of a sequence's last block arrive as zero.
//
// HBM-bound bit copy.  One launch moves every (job, layer, sequence, logical
// block) unit.  The lengths live on the device, so each workgroup derives the
// per-sequence block prefix sums itself (LDS scan over ctx_lens) and then walks
// a grid-strided list of equal-sized 32 KiB work items: no empty workgroups for
// short sequences, no host synchronisation, no scratch memory.  Every lane
// moves 16-byte vectors; a workgroup has four independent 4 KiB loads in flight
// per lane-row before the first store.
#include "kernels.h"
#include "common.hip.h"

namespace fxp {

constexpr int kMoveThreads = 256;
constexpr int kMoveVecPerThread = 8;                                    // 16-byte vectors in flight per lane
constexpr int kMoveChunkBytes = kMoveThreads * 16 * kMoveVecPerThread;  // 32 KiB per work item

__device__ __forceinline__ const char *side_unit_ptr(const KvMoveSide &s, int layer, int seq, int j,
                                                     int blocks_before, int nblk_seq, int64_t unit_bytes)
{
    int64_t unit;
    if (s.table) {
        int32_t phys = s.table[(int64_t)seq * s.max_blocks_per_seq + j];
        unit = (int64_t)(layer - s.layer_base) * s.num_blocks + phys;
    } else {   // packed: [sequence][layer - layer_base][logical block]
        unit = (int64_t)blocks_before * s.n_layers + (int64_t)(layer - s.layer_base) * nblk_seq + j;
    }
    return s.base + unit * unit_bytes;
}

__global__ __launch_bounds__(kMoveThreads) void kv_move_kernel(KvMoveArgs a)
{
    extern __shared__ int32_t prefix[];        // [num_seqs + 1] blocks before each sequence
    __shared__ int32_t part[kMoveThreads];
    const int tid = threadIdx.x;
    const int n = a.num_seqs;

    // ---- exclusive scan of ceil(ctx_len / 16) over the sequences --------------
    const int per = (n + kMoveThreads - 1) / kMoveThreads;
    const int lo = min(tid * per, n), hi = min(lo + per, n);
    int32_t local = 0;
    for (int i = lo; i < hi; ++i) local += (a.ctx_lens[i] + kBlockTokens - 1) / kBlockTokens;
    part[tid] = local;
    __syncthreads();
    if (tid == 0) {
        int32_t run = 0;
        for (int t = 0; t < kMoveThreads; ++t) { int32_t v = part[t]; part[t] = run; run += v; }
        prefix[n] = run;
    }
    __syncthreads();
    {
        int32_t run = part[tid];
        for (int i = lo; i < hi; ++i) { prefix[i] = run; run += (a.ctx_lens[i] + kBlockTokens - 1) / kBlockTokens; }
    }
    __syncthreads();
    const int64_t total_blocks = prefix[n];
    if (total_blocks == 0) return;

    const int64_t unit_bytes = a.unit_bytes;
    const int chunks = (int)((unit_bytes + kMoveChunkBytes - 1) / kMoveChunkBytes);
    const int row_bytes = a.head_dim * 2;                 // one token row of one head
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
        const int j = b - before;
        const int nblk_seq = prefix[seq + 1] - before;
        const int valid = min(kBlockTokens, a.ctx_lens[seq] - j * kBlockTokens);   // valid slots of this block

        const char *sp = side_unit_ptr(job.src, layer, seq, j, before, nblk_seq, unit_bytes);
        char *dp = const_cast<char *>(side_unit_ptr(job.dst, layer, seq, j, before, nblk_seq, unit_bytes));
        if (job.dst.limit_bytes && (dp - job.dst.base) + unit_bytes > job.dst.limit_bytes) continue;   // never past a packed buffer
        if (job.src.limit_bytes && (sp - job.src.base) + unit_bytes > job.src.limit_bytes) continue;

        const int64_t off0 = (int64_t)chunk * kMoveChunkBytes + (int64_t)tid * 16;
        u32x4 v[kMoveVecPerThread];
#pragma unroll
        for (int u = 0; u < kMoveVecPerThread; ++u) {
            const int64_t off = off0 + (int64_t)u * kMoveThreads * 16;
            const int slot = (int)((off / row_bytes) % kBlockTokens);
            v[u] = u32x4{0u, 0u, 0u, 0u};
            if (off < unit_bytes && slot < valid) v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(sp + off));
        }
#pragma unroll
        for (int u = 0; u < kMoveVecPerThread; ++u) {
            const int64_t off = off0 + (int64_t)u * kMoveThreads * 16;
            if (off < unit_bytes) __builtin_nontemporal_store(v[u], reinterpret_cast<u32x4 *>(dp + off));
        }
    }
}

hipError_t launch_kv_move(const KvMoveArgs &args, int grid, hipStream_t stream)
{
    size_t lds = (size_t)(args.num_seqs + 1) * sizeof(int32_t);
    hipLaunchKernelGGL(kv_move_kernel, dim3(grid), dim3(kMoveThreads), lds, stream, args);
    return hipGetLastError();
}

}  // namespace fxp
