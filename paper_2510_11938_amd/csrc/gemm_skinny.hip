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
//     token rows X (<= 128 x K bf16, L2 resident) are the column operand and are
//     re-used across the R tiles;
//   - two register buffers of U k-steps each keep 2*U*R KiB of weights in flight
//     per wavefront while the other buffer is consumed;
//   - split-K across workgroups fills all 256 CUs; partial sums go to a float
//     buffer and are reduced in fixed order by the fused epilogue kernels, so
//     the result is deterministic (no atomics).
#include "kernels.h"
#include "common.hip.h"

namespace fxp {

template <int MT, int R, int U>
__global__ __launch_bounds__(256) void gemm_skinny_kernel(SkinnyArgs a)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int nt0 = (blockIdx.x * 4 + wave) * R;
    if (nt0 >= a.NT) return;
    const int s = blockIdx.y;
    const int ks_begin = (int)((int64_t)a.KS * s / a.S);
    const int ks_end = (int)((int64_t)a.KS * (s + 1) / a.S);

    const u32x4 *wp[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int nt = min(nt0 + r, a.NT - 1);
        wp[r] = reinterpret_cast<const u32x4 *>(a.W) + (int64_t)nt * a.KS * 64 + lane;
    }
    const int mrow = lane & 15, kc = (lane >> 4) * 8;
    const uint16_t *xp[MT];
    bool mvalid[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = mt * 16 + mrow;
        mvalid[mt] = m < a.M;
        xp[mt] = a.X + (int64_t)min(m, a.M - 1) * a.ldx + kc;
    }

    f32x4_t acc[R][MT];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[r][mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    auto load = [&](u32x4(&w)[U][R], u32x4(&x)[U][MT], int ks0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int ks = min(ks0 + u, ks_end - 1);
#pragma unroll
            for (int r = 0; r < R; ++r) w[u][r] = __builtin_nontemporal_load(wp[r] + (int64_t)ks * 64);
            const bool kok = ks * 32 + kc + 8 <= a.K;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                x[u][mt] = u32x4{0u, 0u, 0u, 0u};
                if (mvalid[mt] && kok) x[u][mt] = ld16(xp[mt] + ks * 32);
            }
        }
    };
    auto mma = [&](u32x4(&w)[U][R], u32x4(&x)[U][MT], int ks0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (ks0 + u < ks_end) {
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        acc[r][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            __builtin_bit_cast(bf16x8_t, w[u][r]), __builtin_bit_cast(bf16x8_t, x[u][mt]),
                            acc[r][mt], 0, 0, 0);
            }
        }
    };

    if (ks_begin < ks_end) {
        u32x4 w0[U][R], x0[U][MT], w1[U][R], x1[U][MT];
        load(w0, x0, ks_begin);
        for (int ks = ks_begin; ks < ks_end; ks += 2 * U) {
            if (ks + U < ks_end) load(w1, x1, ks + U);
            mma(w0, x0, ks);
            if (ks + 2 * U < ks_end) load(w0, x0, ks + 2 * U);
            if (ks + U < ks_end) mma(w1, x1, ks + U);
        }
    }

    // accumulator layout of the 16x16 MFMA: lane l, element v holds D[row 4*(l/16)+v][col l%16]
    // with rows = weight rows n and columns = token rows m: four consecutive n per lane.
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
    hipLaunchKernelGGL((gemm_skinny_kernel<MT, R, U>), grid, dim3(256), 0, stream, a);
    return hipGetLastError();
}

template <int MT, int U>
static hipError_t launch_r(const SkinnyArgs &a, hipStream_t stream)
{
    switch (a.R) {
    case 1: return launch_cfg<MT, 1, U>(a, stream);
    case 2: return launch_cfg<MT, 2, U>(a, stream);
    case 4: return launch_cfg<MT, 4, (MT == 8 ? 1 : U)>(a, stream);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_gemm_skinny(const SkinnyArgs &a, hipStream_t stream)
{
    const int mt = (a.M + 15) / 16;
    if (mt <= 1) return launch_r<1, 4>(a, stream);
    if (mt <= 2) return launch_r<2, 4>(a, stream);
    if (mt <= 4) return launch_r<4, 2>(a, stream);
    if (mt <= 8) return launch_r<8, 2>(a, stream);
    return hipErrorInvalidValue;
}

}  // namespace fxp
