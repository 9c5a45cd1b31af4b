// Skinny projection for decode-sized batches (M <= 128 token rows):
//     P[s][m][n] = sum_{k in split s} X[m][k] * W[n][k]
// With a handful of token rows the projection is bound by streaming W from HBM
// (arithmetic intensity ~ M flop per weight byte, far below the machine
// balance), so the kernel is organised around the weight stream:
//   - W is pre-tiled in MFMA operand order (see weight_pack.hip), so every
//     wavefront load of weights is one contiguous 1 KiB, 16 bytes per lane, and
//     goes from HBM straight into the registers that feed
//     v_mfma_f32_16x16x32_bf16 -- no LDS, every weight byte is read once;
//   - each wavefront owns R 16-row tiles of W and a contiguous range of k; the
//     token rows X (<= 128 x K bf16, L2 resident) are the column operand, staged
//     once per workgroup through LDS in operand order (the 4 wavefronts of a
//     workgroup share the k range) and re-used across the R tiles: fetching them
//     per wavefront cost as much L2 bandwidth as the weights themselves;
//   - a ring of NB register buffers of U k-steps each (weights and the token rows
//     of the same group) keeps (NB-1)*U*R KiB of weights in flight per wavefront
//     while one buffer is consumed;
//   - split-K across workgroups fills all 256 CUs; partial sums go to a float
//     buffer and are reduced in fixed order by the fused epilogue kernels, so
//     the result is deterministic (no atomics).  The gate|up projection is wide
//     enough without a split and applies SwiGLU in its own epilogue instead.
#include "kernels.h"
#include "common.hip.h"

namespace fxp {

template <int MT, int R, int U, int NB>
__global__ __launch_bounds__(256) void gemm_skinny_kernel(SkinnyArgs a)
{
    constexpr int kXChunks = U * MT * 64;            // 16-byte chunks of one staged group of token rows
    constexpr int kXPerThread = (kXChunks + 255) / 256;
    __shared__ u32x4 s_x[2][kXChunks];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int nt0 = (blockIdx.x * 4 + wave) * R;
    const int s = blockIdx.y;
    const int ks_begin = (int)((int64_t)a.KS * s / a.S);
    const int ks_end = (int)((int64_t)a.KS * (s + 1) / a.S);
    const int ng = (ks_end - ks_begin + U - 1) / U;  // groups of U k-steps, the last one may be partial

    const u32x4 *wp[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int nt = min(nt0 + r, a.NT - 1);        // tiles past the end are clamped and never stored
        wp[r] = reinterpret_cast<const u32x4 *>(a.W) + packed_operand(nt, 0, a.KS) + lane;
    }

    // Staging of the token rows: chunk q of a group is the 16 bytes that lane q%64 feeds to the
    // MFMA as column operand of (k-step q/64/MT, row tile q/64%MT): row = tile*16 + lane%16,
    // k = step*32 + 8*(lane/16).  Written to LDS in that order, each operand is one linear,
    // conflict-free 1 KiB read, and every token value is fetched from L2 once per workgroup
    // instead of once per wavefront.
    const uint16_t *xsrc[kXPerThread];
    int xstep[kXPerThread], xkc[kXPerThread];
#pragma unroll
    for (int i = 0; i < kXPerThread; ++i) {
        const int q = min(i * 256 + tid, kXChunks - 1);
        const int lane_op = q & 63, t2 = q >> 6;
        const int mt = t2 % MT;
        xstep[i] = t2 / MT;
        xkc[i] = (lane_op >> 4) * 8;
        xsrc[i] = a.X + (int64_t)min(mt * 16 + (lane_op & 15), a.M - 1) * a.ldx + xkc[i];   // rows past M: clamped, never stored
    }

    f32x4_t acc[R][MT];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[r][mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // Everything below is branch-free inside the loop body (indices clamped, invalid k-steps
    // get a zero token operand): a load under a branch makes the compiler's wait-count
    // insertion assume the worst path and drain the prefetch queue before every MFMA group.
    auto load_w = [&](u32x4(&w)[U][R], int g) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int ksc = min(ks_begin + g * U + u, ks_end - 1);
#pragma unroll
            for (int r = 0; r < R; ++r) w[u][r] = __builtin_nontemporal_load(wp[r] + (int64_t)ksc * kPackStepStride);
        }
    };
    // (the zeroing of k-steps past the range happens when the rows are stored to LDS, a group later:
    // a select at load time needs the loaded value at once and would drain the weight prefetch with it)
    auto x_valid = [&](int i, int g) {
        const int ks = ks_begin + g * U + xstep[i];
        return ks < ks_end && ks * 32 + xkc[i] + 8 <= a.K;
    };
    auto load_x = [&](u32x4(&x)[kXPerThread], int g) {
#pragma unroll
        for (int i = 0; i < kXPerThread; ++i) {
            const int ksc = min(ks_begin + g * U + xstep[i], ks_end - 1);
            x[i] = ld16(xsrc[i] + (x_valid(i, g) ? ksc * 32 : 0));
        }
    };
    auto store_x = [&](const u32x4(&x)[kXPerThread], int g, int buf) {
#pragma unroll
        for (int i = 0; i < kXPerThread; ++i)
        {
            const uint32_t keep = x_valid(i, g) ? 0xffffffffu : 0u;      // a mask, not a select: no branch around the store
            const u32x4 v = {x[i].x & keep, x[i].y & keep, x[i].z & keep, x[i].w & keep};
            if (kXChunks % 256 == 0 || i * 256 + tid < kXChunks) s_x[buf][i * 256 + tid] = v;
        }
    };
    auto mma = [&](const u32x4(&w)[U][R], int buf) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            u32x4 xop[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) xop[mt] = s_x[buf][(u * MT + mt) * 64 + lane];
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    acc[r][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        __builtin_bit_cast(bf16x8_t, w[u][r]), __builtin_bit_cast(bf16x8_t, xop[mt]),
                        acc[r][mt], 0, 0, 0);
        }
    };

    // Ring of NB register buffers, weights and token rows alike: the loads of the next NB-1 groups
    // are in flight while one group is multiplied (the products of a group take a tenth of a memory
    // round trip, so two buffers meant one round trip per group).  The token rows of a group are
    // requested together with its weights: the vector-memory counter is in order, and a younger
    // request for rows, waited for before its group's turn, would drain the ring.  The body is
    // unconditional: groups past the end multiply clamped weights by zeroed token rows.
    if (ng > 0) {
        u32x4 w[NB][U][R], xg[NB][kXPerThread];
#pragma unroll
        for (int b = 0; b < NB - 1; ++b) {
            load_w(w[b], b);
            load_x(xg[b], b);
        }
        store_x(xg[0], 0, 0);
        __syncthreads();
        for (int g0 = 0; g0 < ng; g0 += NB) {
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                // weights of group g0+b in w[b], its token rows in s_x[b%2], the rows of the next group in xg[b+1]
                load_w(w[(b + NB - 1) % NB], g0 + b + NB - 1);
                load_x(xg[(b + NB - 1) % NB], g0 + b + NB - 1);
                // keep the requests in front of the group: sunk below the products they would be
                // younger than what the group waits for
                __builtin_amdgcn_sched_barrier(0);
                mma(w[b], b & 1);
                store_x(xg[(b + 1) % NB], g0 + b + 1, (b + 1) & 1);
                __syncthreads();
            }
        }
    }

    // accumulator layout of the 16x16 MFMA: lane l, element v holds D[row 4*(l/16)+v][col l%16]
    // with rows = weight rows n and columns = token rows m: four consecutive n per lane.
    const int mrow = lane & 15;
    if (a.A && a.act == 1) {
        // unsplit projection with relu(sum + bias) in the epilogue
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (nt0 + r >= a.NT) continue;
            const int n = (nt0 + r) * 16 + 4 * (lane >> 4);
            const u32x2 bv = *reinterpret_cast<const u32x2 *>(a.bias + n);
            const float bb[4] = {bf16_lo(bv.x), bf16_hi(bv.x), bf16_lo(bv.y), bf16_hi(bv.y)};
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const int m = mt * 16 + mrow;
                float y[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) y[v] = fmaxf(acc[r][mt][v] + bb[v], 0.f);
                if (m < a.M)
                    *reinterpret_cast<u32x2 *>(a.A + (int64_t)m * a.N + n) = u32x2{pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3])};
            }
        }
        return;
    }
    if constexpr (R % 2 == 0) {
        if (a.A) {
            // gate|up projection without split-K: tiles alternate gate rows / up rows of the same 16
            // features, so the lane that holds a gate value holds the matching up value one tile on
#pragma unroll
            for (int r = 0; r < R; r += 2) {
                if (nt0 + r + 1 >= a.NT) continue;
                const int f = (nt0 + r) / 2 * 16 + 4 * (lane >> 4);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const int m = mt * 16 + mrow;
                    float y[4];
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const float g = acc[r][mt][v];
                        y[v] = g / (1.f + __expf(-g)) * acc[r + 1][mt][v];
                    }
                    if (m < a.M)
                        *reinterpret_cast<u32x2 *>(a.A + (int64_t)m * (a.N / 2) + f) = u32x2{pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3])};
                }
            }
            return;
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        if (nt0 + r >= a.NT) continue;
        const int n = (nt0 + r) * 16 + 4 * (lane >> 4);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int m = mt * 16 + mrow;
            if (m < a.M)
                *reinterpret_cast<f32x4_t *>(a.P + ((int64_t)s * a.M + m) * a.N + n) = acc[r][mt];
        }
    }
}

template <int MT, int R, int U>
static hipError_t launch_cfg(const SkinnyArgs &a, hipStream_t stream)
{
    dim3 grid((a.NT + 4 * R - 1) / (4 * R), a.S);
    constexpr bool kRing4 = MT * R <= 8 && U * R <= 8, kRing8 = MT * R <= 8 && U * R <= 4;    // register budget for four / eight buffers
    if (kRing8 && a.NB >= 8) hipLaunchKernelGGL((gemm_skinny_kernel<MT, R, U, (kRing8 ? 8 : 2)>), grid, dim3(256), 0, stream, a);
    else if (kRing4 && a.NB >= 4) hipLaunchKernelGGL((gemm_skinny_kernel<MT, R, U, (kRing4 ? 4 : 2)>), grid, dim3(256), 0, stream, a);
    else hipLaunchKernelGGL((gemm_skinny_kernel<MT, R, U, 2>), grid, dim3(256), 0, stream, a);
    return hipGetLastError();
}

// a.U = k-steps per register buffer (prefetch depth), rounded down to what is built: 2, 4 or 8,
// and 1 or 2 where four row tiles per wavefront or eight column tiles leave fewer registers
template <int MT, int R>
static hipError_t launch_u(const SkinnyArgs &a, hipStream_t stream)
{
    if constexpr (MT == 8) {
        return R < 4 && a.U >= 2 ? launch_cfg<MT, R, 2>(a, stream) : launch_cfg<MT, R, 1>(a, stream);
    } else if constexpr (R == 4) {
        return MT <= 2 && a.U >= 4 ? launch_cfg<MT, R, 4>(a, stream) : launch_cfg<MT, R, 2>(a, stream);
    } else {
        if (a.U >= 8) return launch_cfg<MT, R, 8>(a, stream);
        if (a.U >= 4) return launch_cfg<MT, R, 4>(a, stream);
        if (a.U >= 2) return launch_cfg<MT, R, 2>(a, stream);
        return launch_cfg<MT, R, 1>(a, stream);
    }
}

template <int MT>
static hipError_t launch_r(const SkinnyArgs &a, hipStream_t stream)
{
    switch (a.R) {
    case 1: return launch_u<MT, 1>(a, stream);
    case 2: return launch_u<MT, 2>(a, stream);
    case 4: return launch_u<MT, 4>(a, stream);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_gemm_skinny(const SkinnyArgs &a, hipStream_t stream)
{
    const int mt = (a.M + 15) / 16;
    if (mt <= 1) return launch_r<1>(a, stream);
    if (mt <= 2) return launch_r<2>(a, stream);
    if (mt <= 4) return launch_r<4>(a, stream);
    if (mt <= 8) return launch_r<8>(a, stream);
    return hipErrorInvalidValue;
}

}  // namespace fxp
