// Re-tiling of a row-major bf16 weight matrix W[N][K] into MFMA operand order.
//
// The projections are evaluated as D[n][m] = sum_k W[n][k] * X[m][k] with the
// weight matrix as the row operand of v_mfma_f32_16x16x32_bf16.  That operand
// wants, per lane l of the wavefront, the 8 consecutive k values
// k0 + 8*(l/16) .. +7 of row n0 + l%16.  Stored in that order,
//     packed[n_tile / 8][k_step][n_tile % 8][lane][8],   n_tile = n/16, k_step = k/32,
// one operand is one contiguous 1 KiB read (16 bytes per lane) and a 128-row
// slab of W is one contiguous stream in the order a workgroup consumes it: the
// layout weight streaming wants when the token count is small and the
// projection is bound by HBM.
//
// K is zero-padded to a multiple of 64.  Rows can be placed at a tile offset
// with a tile stride, which is how Wq|Wk|Wv are concatenated (stride 1) and how
// gate and up rows are interleaved in 16-row tiles (stride 2), so that the
// SwiGLU product needs both halves in the same lane.  For the same reason the row
// tiles of every q and k head are stored with the two halves of the head dimension
// alternating: a rotary pair (d, d + D/2) then sits in one lane of two neighbouring
// accumulator tiles, and a projection can apply the rotation in its own epilogue.
#include "kernels.h"
#include "common.hip.h"

namespace fxp {

__global__ __launch_bounds__(256) void weight_pack_kernel(const uint16_t *__restrict__ src, int N, int K,
                                                          uint16_t *__restrict__ dst, int k_steps,
                                                          int tile_offset, int tile_stride, int half_tiles)
{
    // one thread per 16-byte packed chunk: (n_tile_src, k_step, lane)
    const int64_t total = (int64_t)(N / 16) * k_steps * 64;
    for (int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < total; q += (int64_t)gridDim.x * blockDim.x) {
        const int lane = (int)(q % 64);
        const int ks = (int)((q / 64) % k_steps);
        const int nts = (int)(q / 64 / k_steps);
        const int n = nts * 16 + (lane & 15);
        const int k = ks * 32 + 8 * (lane >> 4);
        u32x4 v = {0u, 0u, 0u, 0u};
        if (k + 8 <= K) v = ld16(src + (int64_t)n * K + k);
        int ntp = nts;                           // position of the source tile among the matrix's tiles
        if (half_tiles > 0) {                    // first-half and second-half tiles of a head alternate (rotary pairs share a lane)
            const int per_head = 2 * half_tiles, j = nts % per_head;
            ntp = nts - j + (j < half_tiles ? 2 * j : 2 * (j - half_tiles) + 1);
        }
        const int64_t ntd = (int64_t)tile_offset + (int64_t)ntp * tile_stride;
        st16(dst + (packed_operand((int)ntd, ks, k_steps) + lane) * 8, v);
    }
}

// a bias vector of the q or k projection in the same tile order as the matrix's rows
__global__ __launch_bounds__(256) void bias_pack_kernel(const uint16_t *__restrict__ src, int n, uint16_t *__restrict__ dst, int half_tiles)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int per_head = 2 * half_tiles, t = i / 16, j = t % per_head;
    const int tp = t - j + (j < half_tiles ? 2 * j : 2 * (j - half_tiles) + 1);
    dst[tp * 16 + i % 16] = src[i];
}

hipError_t launch_bias_pack(const void *src, int n, void *dst, int half_tiles, hipStream_t stream)
{
    hipLaunchKernelGGL(bias_pack_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, static_cast<const uint16_t *>(src), n,
                       static_cast<uint16_t *>(dst), half_tiles);
    return hipGetLastError();
}

hipError_t launch_weight_pack(const void *src, int N, int K, void *dst, int k_steps,
                              int tile_offset, int tile_stride, int half_tiles, hipStream_t stream)
{
    const int64_t total = (int64_t)(N / 16) * k_steps * 64;
    int grid = (int)((total + 255) / 256);
    if (grid > 65535) grid = 65535;
    if (grid < 1) grid = 1;
    hipLaunchKernelGGL(weight_pack_kernel, dim3(grid), dim3(256), 0, stream,
                       static_cast<const uint16_t *>(src), N, K, static_cast<uint16_t *>(dst), k_steps,
                       tile_offset, tile_stride, half_tiles);
    return hipGetLastError();
}

}  // namespace fxp
