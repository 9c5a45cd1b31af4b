// Paged decode attention: one new query token per sequence against the
// sequence's cached keys and values, read through the block table.
//
// Bound by streaming the cache from HBM (every cached K and V byte is read
// exactly once per step, also with grouped query heads: the G query heads of a
// KV head are handled by the same lanes).  Layout of the work:
//   grid  = (context splits, kv heads, sequences); a split is 512 tokens, so
//           long and short contexts give equal-sized workgroups;
//   wave  : takes every 4th 16-token block of the split.  A block's K (and V)
//           for one head is one contiguous 16*D*2-byte run; a wave load
//           instruction covers 1 KiB of it: D/8 lanes per token row, 16 bytes
//           (8 dims) per lane.  The q.k dot product is 8 FMAs per lane plus a
//           log2(D/8)-step butterfly inside the row's lanes.
//   softmax: each group of D/8 lanes keeps its own running (max, sum, acc[8])
//           over the tokens it sees -- no cross-lane traffic in the loop; groups,
//           waves (through LDS) and splits (second kernel) are merged afterwards,
//           always in the same fixed order, so results are bit-reproducible.
//   Two register buffers hold the next block's K and V while the current one is
//   consumed.  Everything after the bf16 loads is float.
#include "kernels.h"
#include "common.hip.h"
#include <math.h>

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

template <int D, int G, bool DEBUG>
__global__ __launch_bounds__(kDecThreads) void attn_decode_kernel(DecodeAttnArgs a)
{
    constexpr int LPT = D / 8;             // lanes per token row
    constexpr int TPI = 64 / LPT;          // token rows per wave load instruction
    constexpr int IPB = kBlockTokens / TPI;  // load instructions per block (K or V)
    constexpr int kBlocksPerSplit = kDecodeSplitTokens / kBlockTokens;

    const int split = blockIdx.x, hk = blockIdx.y, seq = blockIdx.z;
    const int n_keys = a.ctx_lens[seq] + 1;                  // cached tokens + the one appended this step
    const int tok0 = split * kDecodeSplitTokens;
    if (tok0 >= n_keys) return;
    const int nblk = (min(n_keys, tok0 + kDecodeSplitTokens) - tok0 + kBlockTokens - 1) / kBlockTokens;

    __shared__ int32_t s_phys[kBlocksPerSplit];
    __shared__ float s_merge[kDecWaves][G][D + 2];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    if (tid < nblk) s_phys[tid] = a.block_table[(int64_t)seq * a.max_blocks_per_seq + tok0 / kBlockTokens + tid];
    __syncthreads();

    const int dc = lane % LPT, ti = lane / LPT;
    // query, pre-scaled by log2(e)/sqrt(D) so that probabilities are exp2(s - m)
    float q[G][8];
    const int tq = seq;                                       // decode: token index == sequence index
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const u32x4 v = ld16(a.q + ((int64_t)tq * a.n_q_heads + hk * G + g) * D + dc * 8);
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

    const int64_t head_bytes = (int64_t)kBlockTokens * D * 2;
    const int64_t unit_bytes = 2 * (int64_t)a.n_kv_heads * head_bytes;
    const char *layer_base = reinterpret_cast<const char *>(a.pool) + (int64_t)a.layer_local * a.num_blocks * unit_bytes;
    auto load_block = [&](int b, u32x4(&k)[IPB], u32x4(&v)[IPB]) {
        const char *kp = layer_base + (int64_t)s_phys[b] * unit_bytes + (int64_t)hk * head_bytes + lane * 16;
        const char *vp = kp + (int64_t)a.n_kv_heads * head_bytes;
#pragma unroll
        for (int i = 0; i < IPB; ++i) {
            k[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(kp + i * 1024));
            v[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(vp + i * 1024));
        }
    };
    auto consume = [&](int b, const u32x4(&k)[IPB], const u32x4(&v)[IPB]) {
        const int tbase = tok0 + b * kBlockTokens;
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
                        a.dbg_scores[((int64_t)tq * a.n_q_heads + hk * G + g) * a.dbg_stride + tok] = d;
                }
            }
            float mn = m[g];
#pragma unroll
            for (int i = 0; i < IPB; ++i) mn = fmaxf(mn, s[i]);
            const float ms = (mn == -INFINITY) ? 0.f : mn;
            const float alpha = fast_exp2(m[g] - ms);
            m[g] = mn;
            float p[IPB], psum = 0.f;
#pragma unroll
            for (int i = 0; i < IPB; ++i) { p[i] = fast_exp2(s[i] - ms); psum += p[i]; }
            l[g] = l[g] * alpha + psum;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[g][e] *= alpha;
#pragma unroll
            for (int i = 0; i < IPB; ++i) {
                acc[g][0] = fmaf(p[i], bf16_lo(v[i].x), acc[g][0]);
                acc[g][1] = fmaf(p[i], bf16_hi(v[i].x), acc[g][1]);
                acc[g][2] = fmaf(p[i], bf16_lo(v[i].y), acc[g][2]);
                acc[g][3] = fmaf(p[i], bf16_hi(v[i].y), acc[g][3]);
                acc[g][4] = fmaf(p[i], bf16_lo(v[i].z), acc[g][4]);
                acc[g][5] = fmaf(p[i], bf16_hi(v[i].z), acc[g][5]);
                acc[g][6] = fmaf(p[i], bf16_lo(v[i].w), acc[g][6]);
                acc[g][7] = fmaf(p[i], bf16_hi(v[i].w), acc[g][7]);
            }
        }
    };

    {
        u32x4 k0[IPB], v0[IPB], k1[IPB], v1[IPB];
        int b = wave;
        if (b < nblk) load_block(b, k0, v0);
        for (; b < nblk; b += 2 * kDecWaves) {
            const int b1 = b + kDecWaves, b2 = b + 2 * kDecWaves;
            if (b1 < nblk) load_block(b1, k1, v1);
            consume(b, k0, v0);
            if (b2 < nblk) load_block(b2, k0, v0);
            if (b1 < nblk) consume(b1, k1, v1);
        }
    }

    // merge the TPI lane groups of the wave (butterfly: every lane ends with the wave's state)
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int o = LPT; o < 64; o <<= 1) {
            float m2 = __shfl_xor(m[g], o, 64), l2 = __shfl_xor(l[g], o, 64), acc2[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) acc2[e] = __shfl_xor(acc[g][e], o, 64);
            // fixed order: the lower lane group is always the first operand
            if ((lane & o) == 0) merge_state<8>(m[g], l[g], acc[g], m2, l2, acc2);
            else { float mm = m2, ll = l2; merge_state<8>(mm, ll, acc2, m[g], l[g], acc[g]);
                   m[g] = mm; l[g] = ll;
#pragma unroll
                   for (int e = 0; e < 8; ++e) acc[g][e] = acc2[e]; }
        }
        if (ti == 0) {
#pragma unroll
            for (int e = 0; e < 8; ++e) s_merge[wave][g][dc * 8 + e] = acc[g][e];
            if (dc == 0) { s_merge[wave][g][D] = m[g]; s_merge[wave][g][D + 1] = l[g]; }
        }
    }
    __syncthreads();
    // merge the waves in wave order; thread d of the first D threads owns output dim d
    const int n_splits = a.max_splits;
    for (int idx = tid; idx < G * D; idx += kDecThreads) {
        const int g = idx / D, d = idx % D;
        float mm = -INFINITY;
#pragma unroll
        for (int w = 0; w < kDecWaves; ++w) mm = fmaxf(mm, s_merge[w][g][D]);
        const float ms = (mm == -INFINITY) ? 0.f : mm;
        float ll = 0.f, av = 0.f;
#pragma unroll
        for (int w = 0; w < kDecWaves; ++w) {
            const float sc = fast_exp2(s_merge[w][g][D] - ms);
            ll += s_merge[w][g][D + 1] * sc;
            av += s_merge[w][g][d] * sc;
        }
        const int64_t row = ((int64_t)tq * a.n_q_heads + hk * G + g) * n_splits + split;
        a.part_acc[row * D + d] = av;
        if (d == 0) { a.part_ml[row * 2] = mm; a.part_ml[row * 2 + 1] = ll; }
    }
}

// Merge the context splits of each (token, query head) in split order and
// normalise: o = sum_s acc_s 2^(m_s - m) / sum_s l_s 2^(m_s - m).
template <bool DEBUG>
__global__ void attn_decode_combine_kernel(DecodeAttnArgs a)
{
    const int row = blockIdx.x;                      // token * Hq + head
    const int seq = row / a.n_q_heads;
    const int D = a.head_dim;
    const int n_keys = a.ctx_lens[seq] + 1;
    const int ns = (n_keys + kDecodeSplitTokens - 1) / kDecodeSplitTokens;
    const float *ml = a.part_ml + (int64_t)row * a.max_splits * 2;
    float mm = -INFINITY;
    for (int s = 0; s < ns; ++s) mm = fmaxf(mm, ml[s * 2]);
    float ll = 0.f;
    for (int s = 0; s < ns; ++s) ll += ml[s * 2 + 1] * fast_exp2(ml[s * 2] - mm);
    for (int d = threadIdx.x; d < D; d += blockDim.x) {
        float av = 0.f;
        for (int s = 0; s < ns; ++s)
            av += a.part_acc[((int64_t)row * a.max_splits + s) * D + d] * fast_exp2(ml[s * 2] - mm);
        a.out[(int64_t)row * D + d] = f32_to_bf16(av / ll);
    }
    if constexpr (DEBUG) {
        // turn the stored scaled scores (log2 domain) into probabilities
        float *pr = a.dbg_scores + (int64_t)row * a.dbg_stride;
        for (int r = threadIdx.x; r < n_keys; r += blockDim.x) pr[r] = fast_exp2(pr[r] - mm) / ll;
    }
}

template <int D, int G>
static hipError_t launch_dg(const DecodeAttnArgs &a, hipStream_t stream)
{
    dim3 grid(a.max_splits, a.n_kv_heads, a.num_seqs);
    if (a.dbg_scores) hipLaunchKernelGGL((attn_decode_kernel<D, G, true>), grid, dim3(kDecThreads), 0, stream, a);
    else hipLaunchKernelGGL((attn_decode_kernel<D, G, false>), grid, dim3(kDecThreads), 0, stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    dim3 cgrid(a.num_seqs * a.n_q_heads);
    if (a.dbg_scores) hipLaunchKernelGGL(attn_decode_combine_kernel<true>, cgrid, dim3(D), 0, stream, a);
    else hipLaunchKernelGGL(attn_decode_combine_kernel<false>, cgrid, dim3(D), 0, stream, a);
    return hipGetLastError();
}

bool decode_attn_supported(int head_dim, int group)
{
    return (head_dim == 64 || head_dim == 128) && (group == 1 || group == 2 || group == 4 || group == 8);
}

hipError_t launch_attn_decode(const DecodeAttnArgs &a, hipStream_t stream)
{
    const int G = a.n_q_heads / a.n_kv_heads;
#define FXP_DG(DD, GG) if (a.head_dim == DD && G == GG) return launch_dg<DD, GG>(a, stream);
    FXP_DG(128, 1) FXP_DG(128, 2) FXP_DG(128, 4) FXP_DG(128, 8)
    FXP_DG(64, 1) FXP_DG(64, 2) FXP_DG(64, 4) FXP_DG(64, 8)
#undef FXP_DG
    return hipErrorInvalidValue;
}

}  // namespace fxp
