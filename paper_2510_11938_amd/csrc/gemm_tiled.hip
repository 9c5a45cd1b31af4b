// Large-M projection for prefill-sized batches:  C[m][n] = sum_k X[m][k] * W[n][k]
// (+ fused epilogue).  MFMA-bound: v_mfma_f32_16x16x32_bf16, float accumulators.
//
// Workgroup tile: 256 weight rows x 128 token rows, k in steps of 64.
//   - 4 waves stacked along n: each owns 64 weight rows (4 row tiles) and all
//     128 token rows (8 column tiles) -> 32 accumulator tiles, 128 registers;
//   - the weight operand is never shared between waves, and W is stored in
//     MFMA operand order (weight_pack.hip), so it streams HBM/L2 -> registers
//     directly, 1 KiB contiguous per load, one k-step ahead;
//   - the token-row operand is shared by the 4 waves: it is staged through LDS
//     (double buffered, rows padded to 144 bytes so the 16-byte operand reads
//     of 16 consecutive rows hit distinct banks), next tile fetched to registers
//     while the current one is multiplied.
// Epilogues (in registers, each lane holds 4 consecutive n of one token row):
//   plain bf16 store; + residual; SwiGLU over gate/up row tiles interleaved at
//   pack time.
#include "kernels.h"
#include "common.hip.h"

namespace fxp {

constexpr int kTgThreads = 256;
constexpr int kTgBM = 128, kTgBN = 256, kTgBK = 64;
constexpr int kTgRn = 4, kTgRm = 8;
constexpr int kTgPitch = kTgBK * 2 + 16;                 // bytes per LDS row
constexpr int kTgStage = kTgBM * kTgBK / 8 / kTgThreads;  // 16-byte chunks per thread per tile (4)

template <int EPI>
__global__ __launch_bounds__(kTgThreads, 2) void gemm_tiled_kernel(TiledArgs a)
{
    __shared__ __attribute__((aligned(16))) char s_x[2][kTgBM * kTgPitch];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int col = lane & 15, c = lane >> 4;
    const int tiles_n = (a.NT * 16 + kTgBN - 1) / kTgBN;
    const int tile_n = blockIdx.x % tiles_n, tile_m = blockIdx.x / tiles_n;
    const int m0 = tile_m * kTgBM;
    const int nt0 = tile_n * (kTgBN / 16) + wave * kTgRn;     // first 16-row tile of this wave
    const int KT = a.KS / 2;                                   // 64-wide k tiles (K padded to 64)

    const u32x4 *wp[kTgRn];
#pragma unroll
    for (int r = 0; r < kTgRn; ++r)
        wp[r] = reinterpret_cast<const u32x4 *>(a.W) + (int64_t)min(nt0 + r, a.NT - 1) * a.KS * 64 + lane;

    // staging map: chunk q = i*256 + tid -> row q/8, 16-byte chunk q%8 of the 64-wide k tile
    const uint16_t *xsrc[kTgStage];
    int xoff[kTgStage], xk[kTgStage];
#pragma unroll
    for (int i = 0; i < kTgStage; ++i) {
        const int q = i * kTgThreads + tid, r = q >> 3, ch = q & 7;
        xsrc[i] = a.X + (int64_t)min(m0 + r, a.M - 1) * a.ldx + ch * 8;
        xoff[i] = r * kTgPitch + ch * 16;
        xk[i] = ch * 8;
    }

    f32x4_t acc[kTgRn][kTgRm];
#pragma unroll
    for (int r = 0; r < kTgRn; ++r)
#pragma unroll
        for (int mt = 0; mt < kTgRm; ++mt) acc[r][mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    u32x4 xreg[kTgStage], wcur[2][kTgRn], wnext[2][kTgRn];
    auto fetch_x = [&](int kt) {
#pragma unroll
        for (int i = 0; i < kTgStage; ++i) {
            xreg[i] = u32x4{0u, 0u, 0u, 0u};
            if (kt * kTgBK + xk[i] + 8 <= a.K) xreg[i] = ld16(xsrc[i] + kt * kTgBK);
        }
    };
    auto store_x = [&](int buf) {
#pragma unroll
        for (int i = 0; i < kTgStage; ++i) *reinterpret_cast<u32x4 *>(s_x[buf] + xoff[i]) = xreg[i];
    };
    auto fetch_w = [&](u32x4(&w)[2][kTgRn], int kt) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int r = 0; r < kTgRn; ++r) w[h][r] = wp[r][(int64_t)(kt * 2 + h) * 64];
    };

    fetch_x(0);
    fetch_w(wcur, 0);
    store_x(0);
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
        const bool more = kt + 1 < KT;
        if (more) { fetch_x(kt + 1); fetch_w(wnext, kt + 1); }
        const char *xb = s_x[kt & 1];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
#pragma unroll
            for (int mt = 0; mt < kTgRm; ++mt) {
                const u32x4 xop = *reinterpret_cast<const u32x4 *>(xb + (mt * 16 + col) * kTgPitch + h * 64 + c * 16);
#pragma unroll
                for (int r = 0; r < kTgRn; ++r)
                    acc[r][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        __builtin_bit_cast(bf16x8_t, wcur[h][r]), __builtin_bit_cast(bf16x8_t, xop), acc[r][mt], 0, 0, 0);
            }
        }
        if (more) {
            store_x((kt + 1) & 1);
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int r = 0; r < kTgRn; ++r) wcur[h][r] = wnext[h][r];
        }
        __syncthreads();
    }

    // ---- epilogue
#pragma unroll
    for (int mt = 0; mt < kTgRm; ++mt) {
        const int m = m0 + mt * 16 + col;
        if (m >= a.M) continue;
        if constexpr (EPI == kEpiSwiglu) {
#pragma unroll
            for (int r = 0; r < kTgRn; r += 2) {
                if (nt0 + r >= a.NT) continue;          // NT is even and nt0 + r is even: the pair is inside together
                const int f = ((nt0 + r) / 2) * 16 + 4 * c;
                float y[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float g = acc[r][mt][v];
                    y[v] = g / (1.f + __expf(-g)) * acc[r + 1][mt][v];
                }
                *reinterpret_cast<u32x2 *>(a.C + (int64_t)m * a.ldc + f) = u32x2{pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3])};
            }
        } else {
#pragma unroll
            for (int r = 0; r < kTgRn; ++r) {
                if (nt0 + r >= a.NT) continue;
                const int n = (nt0 + r) * 16 + 4 * c;
                float y[4] = {acc[r][mt][0], acc[r][mt][1], acc[r][mt][2], acc[r][mt][3]};
                if constexpr (EPI == kEpiResidual) {
                    const u32x2 rv = *reinterpret_cast<const u32x2 *>(a.R + (int64_t)m * a.ldc + n);
                    y[0] += bf16_lo(rv.x); y[1] += bf16_hi(rv.x); y[2] += bf16_lo(rv.y); y[3] += bf16_hi(rv.y);
                }
                *reinterpret_cast<u32x2 *>(a.C + (int64_t)m * a.ldc + n) = u32x2{pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3])};
            }
        }
    }
}

hipError_t launch_gemm_tiled(const TiledArgs &a, hipStream_t stream)
{
    const int tiles_n = (a.NT * 16 + kTgBN - 1) / kTgBN;
    const int tiles_m = (a.M + kTgBM - 1) / kTgBM;
    dim3 grid(tiles_n * tiles_m);
    switch (a.epilogue) {
    case kEpiStore: hipLaunchKernelGGL(gemm_tiled_kernel<kEpiStore>, grid, dim3(kTgThreads), 0, stream, a); break;
    case kEpiResidual: hipLaunchKernelGGL(gemm_tiled_kernel<kEpiResidual>, grid, dim3(kTgThreads), 0, stream, a); break;
    case kEpiSwiglu: hipLaunchKernelGGL(gemm_tiled_kernel<kEpiSwiglu>, grid, dim3(kTgThreads), 0, stream, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace fxp
