// Row-wise kernels around the projections.  All are HBM/latency bound on tiny
// rows, so each is one pass, 16-byte vectors, one workgroup per token row, and
// each also performs the fixed-order reduction of the split-K partial sums when
// it follows a skinny projection (so no separate reduce launch exists):
//   rmsnorm            n = x * rsqrt(mean(x^2) + eps) * g, or with a norm bias the
//                      LayerNorm n = (x - mean) * rsqrt(var + eps) * g + b
//   qkv_rope_kvwrite   (+ bias,) rotary embedding of q and k at the token's position,
//                      q -> bf16 buffer, rotated k and raw v -> paged cache
//   resid_norm         h = x + proj (+ bias); optionally n = norm(h) for the next block
//   swiglu             a = silu(gate) * up, or relu(sum + bias) for an OPT-style layer
// Sums are float; every value that leaves a kernel is rounded once to bf16.
#include "kernels.h"
#include "common.hip.h"

namespace fxp {

constexpr int kRowThreads = 256;

template <int THREADS = kRowThreads>
__device__ __forceinline__ float block_sum(float v, float *red)
{
    v = wave_sum(v);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    __syncthreads();
    if (lane == 0) red[wave] = v;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < THREADS / 64; ++w) t += red[w];
    return t;
}

__device__ __forceinline__ void unpack8(const u32x4 v, float (&f)[8])
{
    f[0] = bf16_lo(v.x); f[1] = bf16_hi(v.x); f[2] = bf16_lo(v.y); f[3] = bf16_hi(v.y);
    f[4] = bf16_lo(v.z); f[5] = bf16_hi(v.z); f[6] = bf16_lo(v.w); f[7] = bf16_hi(v.w);
}
__device__ __forceinline__ u32x4 pack8(const float (&f)[8])
{
    return u32x4{pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7])};
}
// sum over the S split-K slices of 8 consecutive columns of row t, in slice order.
// The loads of a group of G slices are all issued before the first add (a loop over a
// run-time S issues them one latency after the other); indices past S are clamped to the
// last slice and their values dropped.
template <int G>
__device__ __forceinline__ void partial8_group(const float *P, int S, int s0, int64_t slice_stride, int64_t off, float (&f)[8])
{
    f32x4_t a[G], b[G];
#pragma unroll
    for (int j = 0; j < G; ++j) {
        const float *p = P + (int64_t)min(s0 + j, S - 1) * slice_stride + off;
        a[j] = *reinterpret_cast<const f32x4_t *>(p);
        b[j] = *reinterpret_cast<const f32x4_t *>(p + 4);
    }
#pragma unroll
    for (int j = 0; j < G; ++j) {
        if (s0 + j < S) {
            f[0] += a[j][0]; f[1] += a[j][1]; f[2] += a[j][2]; f[3] += a[j][3];
            f[4] += b[j][0]; f[5] += b[j][1]; f[6] += b[j][2]; f[7] += b[j][3];
        }
    }
}
__device__ __forceinline__ void partial8(const float *P, int S, int64_t slice_stride, int64_t off, float (&f)[8])
{
#pragma unroll
    for (int e = 0; e < 8; ++e) f[e] = 0.f;
    if (S <= 2) partial8_group<2>(P, S, 0, slice_stride, off, f);
    else if (S <= 4) partial8_group<4>(P, S, 0, slice_stride, off, f);
    else for (int s0 = 0; s0 < S; s0 += 8) partial8_group<8>(P, S, s0, slice_stride, off, f);
}

// ---------------------------------------------------------------- rmsnorm / layernorm
// Sum over the row of f(x) by all threads of the workgroup.
template <int THREADS, typename F>
__device__ __forceinline__ float row_reduce(const uint16_t *row, int H, float *red, F f)
{
    float acc = 0.f;
    for (int c = threadIdx.x; c < H / 8; c += THREADS) {
        float v[8];
        unpack8(ld16(row + c * 8), v);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc += f(v[e]);
    }
    return block_sum<THREADS>(acc, red);
}

// The normalisation of one row that is already in memory as bf16: RMSNorm when nb is null,
// LayerNorm (mean removed, variance of the deviations, bias added) otherwise.  ss is the row's
// sum of squares when the caller has it already (RMSNorm only), negative otherwise.
template <int THREADS>
__device__ __forceinline__ void norm_row(const uint16_t *row, const uint16_t *g, const uint16_t *nb, uint16_t *out, int H,
                                         float eps, float ss, float *red)
{
    float mean = 0.f, rstd;
    if (nb) {
        mean = row_reduce<THREADS>(row, H, red, [](float v) { return v; }) / (float)H;
        const float var = row_reduce<THREADS>(row, H, red, [mean](float v) { return (v - mean) * (v - mean); }) / (float)H;
        rstd = rsqrtf(var + eps);
    } else {
        if (ss < 0.f) ss = row_reduce<THREADS>(row, H, red, [](float v) { return v * v; });
        rstd = rsqrtf(ss / (float)H + eps);
    }
    for (int c = threadIdx.x; c < H / 8; c += THREADS) {
        float f[8], gg[8];
        unpack8(ld16(row + c * 8), f);
        unpack8(ld16(g + c * 8), gg);
        if (nb) {
            float bb[8];
            unpack8(ld16(nb + c * 8), bb);
#pragma unroll
            for (int e = 0; e < 8; ++e) f[e] = (f[e] - mean) * rstd * gg[e] + bb[e];
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) f[e] = f[e] * rstd * gg[e];
        }
        st16(out + c * 8, pack8(f));
    }
}

__global__ __launch_bounds__(kRowThreads) void rmsnorm_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ g,
                                                              const uint16_t *__restrict__ b, uint16_t *__restrict__ out, int H, float eps)
{
    __shared__ float red[kRowThreads / 64];
    const int64_t row = (int64_t)blockIdx.x * H;
    norm_row<kRowThreads>(x + row, g, b, out + row, H, eps, -1.f, red);
}

hipError_t launch_rmsnorm(const void *x, const void *g, const void *b, void *out, int T, int H, float eps, hipStream_t stream)
{
    hipLaunchKernelGGL(rmsnorm_kernel, dim3(T), dim3(kRowThreads), 0, stream, static_cast<const uint16_t *>(x),
                       static_cast<const uint16_t *>(g), static_cast<const uint16_t *>(b), static_cast<uint16_t *>(out), H, eps);
    return hipGetLastError();
}

// ---------------------------------------------------------------- residual (+ norm)
// (512 threads at hidden 4096, 1024 above: every thread owns one 8-wide chunk, so all partial-sum
// loads of a row are in flight at once)
template <int THREADS>
__global__ __launch_bounds__(THREADS) void resid_norm_kernel(ResidNormArgs a)
{
    __shared__ float red[THREADS / 64];
    const int t = blockIdx.x;
    const int64_t row = (int64_t)t * a.H;
    if (a.g && !a.nb && a.H / 8 <= THREADS) {
        // RMSNorm behind the residual with at most one 8-wide chunk per thread (every launch of the decode path): the
        // rounded hidden values stay in registers for the norm instead of being read back from the memory they were
        // just stored to (a store, a wait for it, and a second memory round trip in a kernel that is all latency)
        const int c = threadIdx.x;
        const bool live = c < a.H / 8;
        float f[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, gg[8];
        float ss = 0.f;
        if (live) {
            float p[8];
            unpack8(ld16(a.x + row + c * 8), f);
            unpack8(ld16(a.g + c * 8), gg);
            partial8(a.P, a.S, (int64_t)a.T * a.H, row + c * 8, p);
            if (a.bias) {
                float bb[8];
                unpack8(ld16(a.bias + c * 8), bb);
#pragma unroll
                for (int e = 0; e < 8; ++e) p[e] += bb[e];
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) f[e] += p[e];
            const u32x4 hv = pack8(f);
            st16(a.h + row + c * 8, hv);
            unpack8(hv, f);                 // the norm sees the rounded hidden state, as the next stage would
#pragma unroll
            for (int e = 0; e < 8; ++e) ss += f[e] * f[e];
        }
        const float rstd = rsqrtf(block_sum<THREADS>(ss, red) / (float)a.H + a.eps);
        if (live) {
#pragma unroll
            for (int e = 0; e < 8; ++e) f[e] = f[e] * rstd * gg[e];
            st16(a.n + row + c * 8, pack8(f));
        }
        return;
    }
    float ss = 0.f;
    for (int c = threadIdx.x; c < a.H / 8; c += THREADS) {
        float f[8], p[8];
        unpack8(ld16(a.x + row + c * 8), f);
        partial8(a.P, a.S, (int64_t)a.T * a.H, row + c * 8, p);
        if (a.bias) {
            float bb[8];
            unpack8(ld16(a.bias + c * 8), bb);
#pragma unroll
            for (int e = 0; e < 8; ++e) p[e] += bb[e];
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] += p[e];
        const u32x4 hv = pack8(f);
        st16(a.h + row + c * 8, hv);
        unpack8(hv, f);                     // the norm sees the rounded hidden state, as the next stage would
#pragma unroll
        for (int e = 0; e < 8; ++e) ss += f[e] * f[e];
    }
    if (!a.g) return;
    // (every thread reads back only the chunks it wrote itself)
    if (a.nb) norm_row<THREADS>(a.h + row, a.g, a.nb, a.n + row, a.H, a.eps, -1.f, red);
    else norm_row<THREADS>(a.h + row, a.g, nullptr, a.n + row, a.H, a.eps, block_sum<THREADS>(ss, red), red);
}

hipError_t launch_resid_norm(const ResidNormArgs &a, hipStream_t stream)
{
    if (a.H / 8 > 512) hipLaunchKernelGGL(resid_norm_kernel<1024>, dim3(a.T), dim3(1024), 0, stream, a);
    else hipLaunchKernelGGL(resid_norm_kernel<512>, dim3(a.T), dim3(512), 0, stream, a);
    return hipGetLastError();
}

// ---------------------------------------------------------------- SwiGLU
// Gate and up rows were interleaved in 16-row tiles when the weights were
// packed: projection column 32*(f/16) + f%16 is gate row f, +16 is up row f.
__global__ __launch_bounds__(kRowThreads) void swiglu_kernel(SwigluArgs a)
{
    const int t = blockIdx.x;
    const int c = blockIdx.y * kRowThreads + threadIdx.x;       // 8-wide output chunk of row t
    if (c >= a.F / 8) return;
    const int f0 = c * 8;
    float gt[8];
    if (a.act == 1) {                       // relu(sum + bias), columns in natural order
        float bb[8];
        partial8(a.P, a.S, (int64_t)a.T * a.F, (int64_t)t * a.F + f0, gt);
        unpack8(ld16(a.bias + f0), bb);
#pragma unroll
        for (int e = 0; e < 8; ++e) gt[e] = fmaxf(gt[e] + bb[e], 0.f);
    } else {
        const int64_t prow = (int64_t)t * 2 * a.F;
        const int64_t col = 32 * (f0 / 16) + (f0 % 16);
        float up[8];
        partial8(a.P, a.S, (int64_t)a.T * 2 * a.F, prow + col, gt);
        partial8(a.P, a.S, (int64_t)a.T * 2 * a.F, prow + col + 16, up);
#pragma unroll
        for (int e = 0; e < 8; ++e) gt[e] = gt[e] / (1.f + __expf(-gt[e])) * up[e];
    }
    st16(a.out + (int64_t)t * a.ld_out + f0, pack8(gt));
}

hipError_t launch_swiglu(const SwigluArgs &a, hipStream_t stream)
{
    const dim3 grid(a.T, (a.F / 8 + kRowThreads - 1) / kRowThreads);
    hipLaunchKernelGGL(swiglu_kernel, grid, dim3(kRowThreads), 0, stream, a);
    return hipGetLastError();
}

// ---------------------------------------------------------------- RoPE + cache append
// Rotation table of one step: for every token its sequence, its absolute
// position and cos/sin of position * base^(-2d/D), d < D/2.  The angle is
// evaluated in double (it reaches thousands of radians; float would lose the low
// bits before the range reduction).  Positions are the same for every layer of
// the stage, so this runs once per forward call.
constexpr int kRopeTableThreads = kRowThreads;

__global__ __launch_bounds__(kRopeTableThreads) void rope_table_kernel(RopeTableArgs a)
{
    if ((int)blockIdx.x >= a.T) {
        // workgroups past the tokens: the first layer's attention norm, one row each
        __shared__ float red[kRowThreads / 64];
        const int64_t row = (int64_t)(blockIdx.x - a.T) * a.norm_H;
        norm_row<kRowThreads>(a.norm_x + row, a.norm_g, a.norm_b, a.norm_out + row, a.norm_H, a.norm_eps, -1.f, red);
        return;
    }
    __shared__ int s_seq, s_pos;
    const int t = blockIdx.x, half = a.head_dim / 2;
    if (threadIdx.x == 0) {
        // sequence that owns token t: cu[seq] <= t < cu[seq+1] (a chain of dependent loads; a decode step needs none)
        int lo = a.one_token_each ? t : 0, hi = a.one_token_each ? t + 1 : a.num_seqs;
        while (hi - lo > 1) { const int mid = (lo + hi) >> 1; if (a.cu_seqlens_q[mid] <= t) lo = mid; else hi = mid; }
        s_seq = lo;
        s_pos = a.ctx_lens[lo] + (t - a.cu_seqlens_q[lo]);
        a.tok_seq[t] = s_seq;
        a.tok_pos[t] = s_pos;
        a.tok_row[t] = a.block_table[(int64_t)lo * a.max_blocks_per_seq + s_pos / kBlockTokens] * 2 * a.n_kv_heads * kBlockTokens +
                       s_pos % kBlockTokens;
    }
    __syncthreads();
    if ((int)threadIdx.x < half) {
        const double ang = (double)s_pos * pow((double)a.rope_base, -2.0 * (double)threadIdx.x / (double)a.head_dim);
        a.cs[(int64_t)t * half + threadIdx.x] = a.identity ? 1.f : (float)cos(ang);
        a.sn[(int64_t)t * half + threadIdx.x] = a.identity ? 0.f : (float)sin(ang);
    }
    // Workgroup 0 also leaves the exclusive prefix sums of the sequences' cache-block counts
    // (after this step's append), which the decode-attention kernels of every layer cut their
    // work by: each thread sums a contiguous range of sequences, then a log-step scan in LDS.
    if (blockIdx.x == 0) {
        __shared__ int32_t s_scan[kRopeTableThreads];
        const int n = a.num_seqs, nt = kRopeTableThreads, tid = threadIdx.x;
        const int per = (n + nt - 1) / nt;
        const int lo = min(tid * per, n), hi = min(lo + per, n);
        int32_t local = 0;
        // (only the sequences with one new token are the decode kernels' business: in a call that mixes prompt chunks
        // and decode rows the chunks count as zero blocks and go to the prefill kernel)
        auto blocks_of = [&](int i) {
            return a.cu_seqlens_q[i + 1] - a.cu_seqlens_q[i] == 1 ? (a.ctx_lens[i] + 1 + kBlockTokens - 1) / kBlockTokens : 0;
        };
        for (int i = lo; i < hi; ++i) local += blocks_of(i);
        s_scan[tid] = local;
        __syncthreads();
        for (int o = 1; o < nt; o <<= 1) {
            const int32_t v = tid >= o ? s_scan[tid - o] : 0;
            __syncthreads();
            s_scan[tid] += v;
            __syncthreads();
        }
        int32_t run = s_scan[tid] - local;
        for (int i = lo; i < hi; ++i) { a.blk_prefix[i] = run; run += blocks_of(i); }
        if (tid == nt - 1) a.blk_prefix[n] = s_scan[nt - 1];
    }
}

hipError_t launch_rope_table(const RopeTableArgs &a, hipStream_t stream)
{
    hipLaunchKernelGGL(rope_table_kernel, dim3(a.norm_x ? 2 * a.T : a.T), dim3(kRopeTableThreads), 0, stream, a);
    return hipGetLastError();
}

// grid (token, column part): each thread rotates 8 pairs of one q or k head, or
// copies 8 values of a v head; rotated k and v go straight into the token's cache slot.
template <bool FROM_PARTIAL>
__global__ __launch_bounds__(kRowThreads) void qkv_rope_kvwrite_kernel(RopeArgs a)
{
    const int t = blockIdx.x;
    const int D = a.head_dim, half = D / 2;
    const int Nq = a.n_q_heads * D, Nkv = a.n_kv_heads * D, Nall = Nq + 2 * Nkv;
    const int chunks_per_head = half / 8;
    const int n_rot = (a.n_q_heads + a.n_kv_heads) * chunks_per_head, n_v = Nkv / 8;
    const int c = blockIdx.y * kRowThreads + threadIdx.x;
    if (c >= n_rot + n_v) return;
    const int64_t src_row = (int64_t)t * Nall;
    // cache row of (kv, head) for this token: one layer of the pool is [block][K,V][head][16 slots] rows of D values,
    // and the rope table has the token's row for K of head 0
    const int64_t row0 = (int64_t)a.layer_local * a.num_blocks * 2 * a.n_kv_heads * kBlockTokens + a.tok_row[t];

    // col: column of the projection output; q and k heads are in the packed tile order (rotary_col), and so is the bias
    auto fetch8 = [&](int64_t col, float (&f)[8]) {
        if constexpr (FROM_PARTIAL) {
            partial8(a.P, a.S, (int64_t)a.T * Nall, src_row + col, f);
            if (a.bias) {
                float bb[8];
                unpack8(ld16(a.bias + col), bb);
#pragma unroll
                for (int e = 0; e < 8; ++e) f[e] += bb[e];
            }
        } else {
            unpack8(ld16(a.qkv + src_row + col), f);
        }
    };

    if (c < n_rot) {
        const int head = c / chunks_per_head, d0 = (c % chunks_per_head) * 8;
        float lo[8], hi[8], rl[8], rh[8];
        fetch8(rotary_col(head * D, d0, D), lo);
        fetch8(rotary_col(head * D, d0 + half, D), hi);
        const float *cs = a.cs + (int64_t)t * half + d0, *sn = a.sn + (int64_t)t * half + d0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float co = cs[e], si = sn[e];
            rl[e] = lo[e] * co - hi[e] * si;
            rh[e] = hi[e] * co + lo[e] * si;
        }
        uint16_t *dst;
        if (head < a.n_q_heads) dst = a.q_out + (int64_t)t * Nq + (int64_t)head * D;
        else dst = a.pool + (row0 + (int64_t)(head - a.n_q_heads) * kBlockTokens) * D;
        st16(dst + d0, pack8(rl));
        st16(dst + d0 + half, pack8(rh));
    } else {
        const int cv = c - n_rot;
        const int head = (cv * 8) / D, d0 = (cv * 8) % D;
        float f[8];
        fetch8((int64_t)Nq + Nkv + cv * 8, f);
        st16(a.pool + (row0 + (int64_t)(a.n_kv_heads + head) * kBlockTokens) * D + d0, pack8(f));
    }
}

hipError_t launch_qkv_rope_kvwrite(const RopeArgs &a, hipStream_t stream)
{
    const int chunks = (a.n_q_heads + a.n_kv_heads) * (a.head_dim / 16) + a.n_kv_heads * a.head_dim / 8;
    const dim3 grid(a.T, (chunks + kRowThreads - 1) / kRowThreads);
    if (a.P) hipLaunchKernelGGL(qkv_rope_kvwrite_kernel<true>, grid, dim3(kRowThreads), 0, stream, a);
    else hipLaunchKernelGGL(qkv_rope_kvwrite_kernel<false>, grid, dim3(kRowThreads), 0, stream, a);
    return hipGetLastError();
}

}  // namespace fxp
