// Large-M projection for prefill-sized batches:  C[m][n] = sum_k X[m][k] * W[n][k]
// (+ fused epilogue).  MFMA-bound: v_mfma_f32_16x16x32_bf16, float accumulators.
//
// Workgroup tile: 256 weight rows x 128 token rows, k in steps of 32 (one MFMA k-step).
//   - 4 waves stacked along n: each owns 64 weight rows (4 row tiles) and all
//     128 token rows (8 column tiles) -> 32 accumulator tiles, 128 registers;
//   - the weight operand is never shared between waves, and W is stored in
//     MFMA operand order (weight_pack.hip), so it streams L2 -> registers
//     directly, 1 KiB contiguous per load, through a 3-deep register ring
//     (loads issued one k-step before use, spread over the stage);
//   - the token-row operand is shared by the 4 waves: it goes global -> registers
//     -> LDS in stages of 64 k (two k-steps), fetched two stages ahead with full
//     128-byte lines per row, and is stored in MFMA operand order with a slot
//     swizzle so that both the staging writes and the linear-by-lane operand
//     reads are free of bank conflicts; three LDS buffers, one barrier per stage;
//   - the 32 MFMAs of a k-step are four inline-assembly blocks, each of which
//     requests the operand pair of the next block before multiplying its own;
//     the chain continues across k-steps and stages (the next stage's rows are
//     already in LDS), so no MFMA waits for a cold LDS read;
//   - every load is unconditional (clamped index + select): a load under a branch
//     makes the compiler drain the whole prefetch queue at the next wait.
// Workgroups are numbered so that the 32 that run together on one XCD (they share
// an L2) form a 4 x 8 block of tiles and walk k in step: each weight k-slice is
// fetched into that L2 once per 8 workgroups, each token k-slice once per 4.
// Epilogues (in registers, each lane holds 4 consecutive n of one token row):
//   plain bf16 store; + residual; SwiGLU over gate/up row tiles interleaved at
//   pack time; float partial sums of a k range (grid.y = split-K factor), used for
//   decode batches of 65..128 tokens where one 128-row tile covers the batch and
//   the k split supplies the parallelism.
#include "kernels.h"
#include <stdlib.h>
#include "common.hip.h"

namespace fxp {

constexpr int kTgThreads = 256;
constexpr int kTgBM = 128, kTgBN = 256;
constexpr int kTgRn = 4, kTgRm = 8;
constexpr int kTgStages = 3;                               // LDS buffers, each one stage of two k-steps (64 k)
constexpr int kTgXChunks = 2 * kTgRm * 64;                 // 16-byte chunks of one stage (16 KiB)
constexpr int kTgXPerThread = kTgXChunks / kTgThreads;     // 4

template <int EPI, bool K_TAIL, bool W_EARLY>
__global__ __launch_bounds__(kTgThreads, 2) void gemm_tiled_kernel(TiledArgs a)
{
    __shared__ u32x4 s_x[kTgStages][kTgXChunks];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int col = lane & 15, c = lane >> 4;

    // ---- tile of this workgroup (XCD-aware numbering, see the header comment)
    const int tiles_n = (a.NT * 16 + kTgBN - 1) / kTgBN, tiles_m = (a.M + kTgBM - 1) / kTgBM;
    int tile_m, tile_n;
    if (tiles_m == 1) {          // one row of tiles (at most 128 token rows): nothing to share but the token rows
        tile_m = 0;
        tile_n = blockIdx.x;
    } else if (tiles_m < 16) {
        // up to 15 rows of tiles: XCD x takes the weight tiles n = x mod 8 and walks the token tiles of each in turn,
        // so the workgroups that share weight rows follow each other on one L2
        const int xcd = blockIdx.x % kXcds, seq = blockIdx.x / kXcds;
        tile_m = seq % tiles_m;
        tile_n = (seq / tiles_m) * kXcds + xcd;
    } else {
        constexpr int kBlkN = 4, kBlkM = 8;                 // 32 workgroups of one XCD = 4 x 8 tiles
        const int blocks_n = (tiles_n + kBlkN - 1) / kBlkN;
        const int id = blockIdx.x;
        const int xcd = id % kXcds, seq = id / kXcds;          // seq-th workgroup given to this XCD
        const int super = seq / (kBlkN * kBlkM), within = seq % (kBlkN * kBlkM);
        const int sb = super * kXcds + xcd;                   // super-block index
        tile_n = (sb % blocks_n) * kBlkN + within % kBlkN;
        tile_m = (sb / blocks_n) * kBlkM + within / kBlkN;
    }
    if (tile_n >= tiles_n || tile_m >= tiles_m) return;
    const int m0 = tile_m * kTgBM;
    const int nt0 = tile_n * (kTgBN / 16) + wave * kTgRn;     // first 16-row tile of this wave
    const int KS = a.KS;

    const u32x4 *wp[kTgRn];
#pragma unroll
    for (int r = 0; r < kTgRn; ++r)
        wp[r] = reinterpret_cast<const u32x4 *>(a.W) + packed_operand(min(nt0 + r, a.NT - 1), 0, KS) + lane;

    // Staging map.  Global side: chunk q = i*256 + tid is 16 bytes of token row q/8, k-chunk q%8
    // of the 64-wide stage, so 8 consecutive lanes fetch one full 128-byte line (a wave
    // instruction that touches 16 rows with 64 bytes each, as the operand order would have it,
    // costs twice the cache-line requests and was the largest stall of this kernel).
    // LDS side: the chunk belongs to k-step h = (q%8)/4, column tile mt = row/16, operand lane
    // (m16 = row%16, c = (q%8)%4).  Inside the 1 KiB operand block it is stored at slot
    // 16*c + ((m16 + 2*c + 8*h) & 15): a bijection per block, so the linear-by-lane operand
    // reads stay conflict-free, and the 16 lanes of one LDS write cycle (2 rows x 8 chunks)
    // hit 16 different 16-byte bank groups.
    const uint16_t *xsrc[kTgXPerThread];
    int xdst[kTgXPerThread], xkc[kTgXPerThread];
#pragma unroll
    for (int i = 0; i < kTgXPerThread; ++i) {
        const int q = i * kTgThreads + tid, row = q >> 3, ch = q & 7;
        const int h = ch >> 2, cc = ch & 3, mt = row >> 4, m16 = row & 15;
        xkc[i] = ch * 8;
        xsrc[i] = a.X + (int64_t)min(m0 + row, a.M - 1) * a.ldx + xkc[i];
        xdst[i] = (h * kTgRm + mt) * 64 + 16 * cc + ((m16 + 2 * cc + 8 * h) & 15);
    }

    f32x4_t acc[kTgRn][kTgRm];
#pragma unroll
    for (int r = 0; r < kTgRn; ++r)
#pragma unroll
        for (int mt = 0; mt < kTgRm; ++mt) acc[r][mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // stages of 64 k (K is padded to 64); split s of S owns stages [kt0, kt0 + KT)
    const int kt0 = (int)((int64_t)(KS / 2) * blockIdx.y / gridDim.y);
    const int KT = (int)((int64_t)(KS / 2) * (blockIdx.y + 1) / gridDim.y) - kt0;
    auto fetch_w = [&](u32x4(&w)[kTgRn], int ks) {
        const int ksc = 2 * kt0 + min(ks, 2 * KT - 1);
#pragma unroll
        for (int r = 0; r < kTgRn; ++r) w[r] = wp[r][(int64_t)ksc * kPackStepStride];
    };
    auto fetch_x = [&](u32x4(&x)[kTgXPerThread], int kt) {
        const int ktc = kt0 + min(kt, KT - 1);
#pragma unroll
        for (int i = 0; i < kTgXPerThread; ++i) {
            if constexpr (K_TAIL) {                         // K not a multiple of 64: zero operand past the end
                const bool ok = ktc * 64 + xkc[i] + 8 <= a.K;
                const u32x4 v = ld16(xsrc[i] + (ok ? ktc * 64 : 0));
                x[i] = ok ? v : u32x4{0u, 0u, 0u, 0u};
            } else {
                x[i] = ld16(xsrc[i] + ktc * 64);
            }
        }
    };
    auto store_x = [&](const u32x4(&x)[kTgXPerThread], int stage) {
#pragma unroll
        for (int i = 0; i < kTgXPerThread; ++i) s_x[stage][xdst[i]] = x[i];
    };
    // One k-step of the wave tile: 8 column-tile operands from LDS, 32 MFMAs, written as four
    // inline-assembly blocks of 8 MFMAs (two column tiles) because the compiler's scheduler puts
    // every LDS read directly in front of its first use and then waits for it, which leaves the
    // matrix pipe idle for the LDS latency.  Every block first issues the LDS reads of the operand
    // pair that the NEXT block multiplies and then waits only for its own pair (lgkmcnt(2):
    // everything but the two reads just issued; LDS returns in order), which was requested one
    // block earlier.  The chain runs across k-steps and across stages: the last block of a k-step
    // requests the first pair of the next one (the token rows of the next stage are already in
    // LDS, see below), so the pipe never waits for a cold LDS read after the prologue.
    // Two operand register sets (A, B) alternate; four blocks per k-step keep their roles fixed.
#define FXP_MFMA8(X0, X1)                                                  \
    "v_mfma_f32_16x16x32_bf16 %[a0], %[w0], %[" #X0 "], %[a0]\n"              \
    "v_mfma_f32_16x16x32_bf16 %[a1], %[w1], %[" #X0 "], %[a1]\n"              \
    "v_mfma_f32_16x16x32_bf16 %[a2], %[w2], %[" #X0 "], %[a2]\n"              \
    "v_mfma_f32_16x16x32_bf16 %[a3], %[w3], %[" #X0 "], %[a3]\n"              \
    "v_mfma_f32_16x16x32_bf16 %[b0], %[w0], %[" #X1 "], %[b0]\n"              \
    "v_mfma_f32_16x16x32_bf16 %[b1], %[w1], %[" #X1 "], %[b1]\n"              \
    "v_mfma_f32_16x16x32_bf16 %[b2], %[w2], %[" #X1 "], %[b2]\n"              \
    "v_mfma_f32_16x16x32_bf16 %[b3], %[w3], %[" #X1 "], %[b3]\n"
#define FXP_ACC8(M)                                                                  \
    [a0] "+v"(acc[0][M]), [a1] "+v"(acc[1][M]), [a2] "+v"(acc[2][M]), [a3] "+v"(acc[3][M]),         \
    [b0] "+v"(acc[0][M + 1]), [b1] "+v"(acc[1][M + 1]), [b2] "+v"(acc[2][M + 1]), [b3] "+v"(acc[3][M + 1])
#define FXP_WOPS [w0] "v"(w[0]), [w1] "v"(w[1]), [w2] "v"(w[2]), [w3] "v"(w[3])
    // request column tiles (OFF0, OFF1) at NADDR into (N0, N1); multiply column tiles M, M+1 held in (C0, C1)
#define FXP_BLOCK(N0, N1, NADDR, OFF0, OFF1, C0, C1, M)                                              \
    asm volatile("ds_read_b128 %[n0], %[naddr] offset:" #OFF0 "\n"                                    \
                 "ds_read_b128 %[n1], %[naddr] offset:" #OFF1 "\n"                                    \
                 "s_waitcnt lgkmcnt(2)\n" FXP_MFMA8(c0, c1)                                            \
                 : [n0] "=&v"(N0), [n1] "=&v"(N1), FXP_ACC8(M)                                        \
                 : [naddr] "v"(NADDR), FXP_WOPS, [c0] "v"(C0), [c1] "v"(C1)                           \
                 : "memory");
    u32x4 xa0, xa1, xb0, xb1;          // operand sets A and B
    // lds_addr: this lane's 16 bytes of column tile 0 of the k-step (tile t is 1 KiB further per t);
    // next_addr: the same for the k-step that follows.  On entry set A holds (or is about to
    // receive) column tiles 0, 1 of this k-step; on exit it has been asked for those of the next.
    auto compute = [&](const u32x4(&w)[kTgRn], uint32_t lds_addr, uint32_t next_addr) {
        FXP_BLOCK(xb0, xb1, lds_addr, 2048, 3072, xa0, xa1, 0)
        FXP_BLOCK(xa0, xa1, lds_addr, 4096, 5120, xb0, xb1, 2)
        FXP_BLOCK(xb0, xb1, lds_addr, 6144, 7168, xa0, xa1, 4)
        FXP_BLOCK(xa0, xa1, next_addr, 0, 1024, xb0, xb1, 6)
    };
#undef FXP_BLOCK
#undef FXP_MFMA8
#undef FXP_ACC8
#undef FXP_WOPS
    // byte address in LDS of this lane's operand slot of column tile 0, for k-step half h of stage 0
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)(&s_x[0][0]);
    const uint32_t lds_h0 = lds_base + (16 * c + ((col + 2 * c) & 15)) * 16;
    const uint32_t lds_h1 = lds_base + (kTgRm * 64 + 16 * c + ((col + 2 * c + 8) & 15)) * 16;
    constexpr uint32_t kStageBytes = kTgXChunks * 16;

    // Weights: ring of three k-steps.  With many row tiles (matrix-core bound) w(ks+2) is requested after the
    // products of k-step ks, one k-step ahead of its use, and not together with the token rows at the start of
    // the stage: requests spread evenly over the stage measured 4 % faster than the same loads in one burst a
    // k-step earlier (placements between the two were all within 1 % of this one).  With one or two row tiles
    // (W_EARLY: the launch streams the weights once and is bound by HBM) the earlier request keeps more bytes
    // in flight and is the faster one (70B shape, 256 rows: 305 against 318 us per layer).  Token rows:
    // three LDS buffers; stage t+2 is fetched to registers at the start of stage t and written to
    // buffer (t+2) % 3 at its end.  That buffer was last read in stage t-1, so the one barrier per
    // stage (at its end) orders those reads before these writes, and it makes the rows of stage
    // t+1, written a stage earlier, visible before the last block of stage t asks for them.
    // Three stages (six k-steps) per trip so that every register set and buffer keeps its name.
    u32x4 w0[kTgRn], w1[kTgRn], w2[kTgRn], xg[kTgXPerThread];
    fetch_x(xg, 0);
    fetch_w(w0, 0);
    fetch_w(w1, 1);
    store_x(xg, 0);
    fetch_x(xg, 1);
    store_x(xg, 1);
    __syncthreads();
    asm volatile("ds_read_b128 %[n0], %[addr]\n"
                 "ds_read_b128 %[n1], %[addr] offset:1024\n"
                 : [n0] "=&v"(xa0), [n1] "=&v"(xa1) : [addr] "v"(lds_h0) : "memory");
#define FXP_TG_STAGE(WA, WB, WC2, WD2, KTV, BUF, BUF_NEXT, BUF_STORE)          \
    fetch_x(xg, (KTV) + 2);                                                    \
    if constexpr (W_EARLY) fetch_w(WC2, 2 * (KTV) + 2);                        \
    compute(WA, lds_h0 + (BUF) * kStageBytes, lds_h1 + (BUF) * kStageBytes);   \
    if constexpr (W_EARLY) fetch_w(WD2, 2 * (KTV) + 3); else fetch_w(WC2, 2 * (KTV) + 2); \
    compute(WB, lds_h1 + (BUF) * kStageBytes, lds_h0 + (BUF_NEXT) * kStageBytes); \
    if constexpr (!W_EARLY) fetch_w(WD2, 2 * (KTV) + 3);                       \
    store_x(xg, BUF_STORE);                                                    \
    __syncthreads();
    // k-step s lives in weight set s % 3 and stage t in LDS buffer t % 3, so the names repeat every three stages
    int kt = 0;
    for (; kt + 3 <= KT; kt += 3) {
        FXP_TG_STAGE(w0, w1, w2, w0, kt, 0, 1, 2)          // k-steps 6j,   6j+1; fetches w(6j+2) -> w2, w(6j+3) -> w0
        FXP_TG_STAGE(w2, w0, w1, w2, kt + 1, 1, 2, 0)      // k-steps 6j+2, 6j+3; fetches w(6j+4) -> w1, w(6j+5) -> w2
        FXP_TG_STAGE(w1, w2, w0, w1, kt + 2, 2, 0, 1)      // k-steps 6j+4, 6j+5; fetches w(6j+6) -> w0, w(6j+7) -> w1
    }
    if (kt < KT) {
        FXP_TG_STAGE(w0, w1, w2, w0, kt, 0, 1, 2)
        if (kt + 1 < KT) { FXP_TG_STAGE(w2, w0, w1, w2, kt + 1, 1, 2, 0) }
    }
    // the last block's request for a further k-step is never used, but its registers must not be
    // given to anything else before the data has landed
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(xa0), "+v"(xa1) : : "memory");
#undef FXP_TG_STAGE

    // ---- epilogue.  A wait for a load also waits for the stores before it (one counter), and the compiler waits for a
    // load right where it is used, so loads scattered between the stores make a chain of round trips at the end of a
    // tile: the bias is read once and the residual (which may be the output buffer itself: no load can be moved across a
    // store; a lane reads only the addresses it writes itself) for four token tiles at a time, ahead of their stores.
    u32x2 bias_v[kTgRn];
#pragma unroll
    for (int r = 0; r < kTgRn; ++r)
        bias_v[r] = (EPI != kEpiPartial && EPI != kEpiSwiglu && a.bias) ? *reinterpret_cast<const u32x2 *>(a.bias + min(nt0 + r, a.NT - 1) * 16 + 4 * c)
                                                                        : u32x2{0u, 0u};
    constexpr int kGroup = 4;
#pragma unroll
    for (int mg = 0; mg < kTgRm; mg += kGroup) {
        u32x2 resid[kGroup][kTgRn];
        if constexpr (EPI == kEpiResidual) {
#pragma unroll
            for (int g = 0; g < kGroup; ++g)
#pragma unroll
                for (int r = 0; r < kTgRn; ++r)
                    resid[g][r] = *reinterpret_cast<const u32x2 *>(a.R + (int64_t)min(m0 + (mg + g) * 16 + col, a.M - 1) * a.ldc +
                                                                   min(nt0 + r, a.NT - 1) * 16 + 4 * c);
        }
#pragma unroll
        for (int g = 0; g < kGroup; ++g) {
            const int mt = mg + g;
            const int m = m0 + mt * 16 + col;
            if (m >= a.M) continue;
            if constexpr (EPI == kEpiPartial) {
#pragma unroll
                for (int r = 0; r < kTgRn; ++r) {
                    if (nt0 + r >= a.NT) continue;
                    const int n = (nt0 + r) * 16 + 4 * c;
                    *reinterpret_cast<f32x4_t *>(a.P + ((int64_t)blockIdx.y * a.M + m) * (a.NT * 16) + n) = acc[r][mt];
                }
            } else if constexpr (EPI == kEpiSwiglu) {
#pragma unroll
                for (int r = 0; r < kTgRn; r += 2) {
                    if (nt0 + r >= a.NT) continue;          // NT is even and nt0 + r is even: the pair is inside together
                    const int f = ((nt0 + r) / 2) * 16 + 4 * c;
                    float y[4];
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const float gt = acc[r][mt][v];
                        y[v] = gt / (1.f + __expf(-gt)) * acc[r + 1][mt][v];
                    }
                    *reinterpret_cast<u32x2 *>(a.C + (int64_t)m * a.ldc + f) = u32x2{pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3])};
                }
            } else {
#pragma unroll
                for (int r = 0; r < kTgRn; ++r) {
                    if (nt0 + r >= a.NT) continue;
                    const int n = (nt0 + r) * 16 + 4 * c;
                    float y[4] = {acc[r][mt][0] + bf16_lo(bias_v[r].x), acc[r][mt][1] + bf16_hi(bias_v[r].x),
                                  acc[r][mt][2] + bf16_lo(bias_v[r].y), acc[r][mt][3] + bf16_hi(bias_v[r].y)};
                    if constexpr (EPI == kEpiRelu) {
#pragma unroll
                        for (int v = 0; v < 4; ++v) y[v] = fmaxf(y[v], 0.f);
                    }
                    if constexpr (EPI == kEpiResidual) {
                        const u32x2 rv = resid[g][r];
                        y[0] += bf16_lo(rv.x); y[1] += bf16_hi(rv.x); y[2] += bf16_lo(rv.y); y[3] += bf16_hi(rv.y);
                    }
                    *reinterpret_cast<u32x2 *>(a.C + (int64_t)m * a.ldc + n) = u32x2{pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3])};
                }
            }
        }
    }
}


// ---------------------------------------------------------------------------------------------------------
// Wide tile for matrix-core-bound launches (thousands of token rows): 256 weight rows x 256 token rows per
// workgroup, ONE workgroup of four waves per CU.  Each wave owns 64 weight rows and all 256 token rows: 64
// accumulator tiles in the 256 accumulation registers.  Against the 256 x 128 tile above this halves the weight
// bytes a CU has to pull in per product (128 B instead of 192 B per MFMA through the 64 B/clk vector-memory path,
// which was what bounded that kernel at two thirds of the matrix cores).
//   - weights: still straight from global memory into registers in operand order (never through LDS), requested
//     three stages (six k-steps) ahead into a ring of four register sets;
//   - token rows: global -> LDS directly (16-byte LDS-DMA loads, no registers, no LDS store instructions), three
//     stages ahead, four LDS buffers of one 64-wide stage each (32 KiB).  One DMA instruction brings eight full
//     128-byte rows; the data lands in lane order, so the LDS image is row-major with 128 bytes per row, and the
//     swizzle that keeps the operand reads conflict-free is applied on the GLOBAL side: the lane that fills
//     16-byte position p of row r fetches chunk p ^ ((r >> 1) & 7) of that row (measured: no bank conflicts);
//   - with one wave per SIMD nothing else covers a wave's stalls or the issue time of its own loads, so the main
//     loop is hand-placed: blocks of eight MFMAs, each with the two LDS reads of the operand pair of the block
//     THREE further on and one load of the stage (sixteen blocks, sixteen loads) issued between its products,
//     wave-uniform load addresses in scalar registers so that a load is one instruction, and every wait written
//     by hand (the compiler, left to count the loads, drained them where a stage first touched its weights).
//     Measured on the way, 7B gate|up projection at 15,928 rows: loads as compiler statements between the blocks
//     and reads one block ahead 1.33 PFLOP/s (the 256 x 128 tile: 1.30); reads three blocks ahead between the
//     products 1.41; loads inside the blocks 1.50; the same loop without any load 1.70.
// Requirements (else the kernel above is used): at least 1024 token rows, K a multiple of 256, whole 64-row wave
// tiles, token-row byte offsets below 4 GiB; and the launcher's estimate that this tile is the faster one for the
// launch's tile counts (wide_tile_fits).
constexpr int kWdBM = 256, kWdBN = 256, kWdRn = 4, kWdRm = 16, kWdBufs = 4;
constexpr int kWdStageBytes = kWdBM * 128;                 // 256 rows x 64 k of bf16
constexpr int kWdLdsBytes = kWdBufs * kWdStageBytes;       // 128 KiB

// PROBE != 0 (tuning builds only; results are wrong on purpose, every access that remains is unchanged): the main loop
// without its loads, i.e. what the LDS reads and the products alone take.
template <int EPI, int PROBE = 0>
__global__ __launch_bounds__(kTgThreads, 1) void gemm_wide_kernel(TiledArgs a)
{
    extern __shared__ __attribute__((aligned(1024))) char s_wide[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 15, c = lane >> 4;

    // ---- tile of this workgroup: the 32 workgroups of one XCD (one per CU) form a super-block of (32 / blk_m) x blk_m
    // tiles that share weight and token rows in that XCD's L2; the launcher picks the shape that wastes the fewest slots
    const int tiles_n = (a.NT * 16 + kWdBN - 1) / kWdBN, tiles_m = (a.M + kWdBM - 1) / kWdBM;
    int tile_m, tile_n;
    {
        const int blk_m = a.blk_m, blk_n = 32 / blk_m;
        const int blocks_n = (tiles_n + blk_n - 1) / blk_n;
        const int id = blockIdx.x;
        const int xcd = id % kXcds, seq = id / kXcds;
        const int super = seq / 32, within = seq % 32;
        const int sb = super * kXcds + xcd;
        tile_n = (sb % blocks_n) * blk_n + within % blk_n;
        tile_m = (sb / blocks_n) * blk_m + within / blk_n;
    }
    if (tile_n >= tiles_n || tile_m >= tiles_m) return;
    const int m0 = tile_m * kWdBM;
    const int nt0 = tile_n * (kWdBN / 16) + wave * kWdRn;      // first 16-row tile of this wave (a multiple of 4)
    const int KS = a.KS, KT = KS / 2;                          // stages of 64 k

    // Loads are issued from inside the inline-assembly blocks of the main loop (below), with a wave-uniform base address
    // in scalar registers plus a constant per-lane offset, so that a load costs one instruction and no address arithmetic
    // in the vector pipe, and the compiler keeps no account of them: every wait is placed by hand.
    // weights of this wave: tiles nt0 .. nt0+3 lie in one group of the packed layout, 1 KiB apart; k-steps 8 KiB apart
    const char *wbase = reinterpret_cast<const char *>(a.W) + packed_operand(min(nt0, a.NT - kWdRn), 0, KS) * 16;
    const uint32_t wlane = lane * 16;
    auto wptr = [&](int ks) { return wbase + (int64_t)min(ks, KS - 1) * (kPackStepStride * 16); };
    // token rows: DMA instruction i of this wave brings rows wave*64 + 8i .. +7 of the stage (lane / 8 = row, lane % 8 =
    // position in the row); source chunk = position ^ swizzle(row); byte offsets fit 32 bits (checked by the launcher)
    uint32_t xoff[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int row = wave * 64 + i * 8 + (lane >> 3);
        const int chunk = (lane & 7) ^ ((row >> 1) & 7);
        xoff[i] = (uint32_t)min(m0 + row, a.M - 1) * (uint32_t)(a.ldx * 2) + chunk * 16;      // rows past the end: clamped, never stored
    }
    const char *xbase = reinterpret_cast<const char *>(a.X);
    auto xptr = [&](int kt) { return xbase + (int64_t)min(kt, KT - 1) * 128; };
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)s_wide;
    const uint32_t lds_dma = lds_base + wave * (64 * 128);          // this wave's rows inside a stage buffer

    f32x4_t acc[kWdRn][kWdRm];
#pragma unroll
    for (int r = 0; r < kWdRn; ++r)
#pragma unroll
        for (int mt = 0; mt < kWdRm; ++mt) acc[r][mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // operand reads: lane (col, c) of column tile mt, k-step half h reads row mt*16 + col, chunk 4h + c
    const int sw = (col >> 1) & 7;
    const uint32_t lds_h0 = lds_base + (col * 8 + (c ^ sw)) * 16;
    const uint32_t lds_h1 = lds_base + (col * 8 + ((4 + c) ^ sw)) * 16;

#define FXP_ACC8(M)                                                                  \
    [a0] "+a"(acc[0][M]), [a1] "+a"(acc[1][M]), [a2] "+a"(acc[2][M]), [a3] "+a"(acc[3][M]),         \
    [b0] "+a"(acc[0][M + 1]), [b1] "+a"(acc[1][M + 1]), [b2] "+a"(acc[2][M + 1]), [b3] "+a"(acc[3][M + 1])
    // One block: the eight MFMAs of column tiles M, M+1 (operands in C0, C1, asked for three blocks earlier) with the two
    // LDS reads of the operand pair of the block three further on (NADDR + OFF0, OFF1 -> N0, N1) and one load of the
    // stage (XPRE: the M0 write of a DMA load, one product ahead of it; XASM: the load) issued between its products,
    // where they cost the matrix cores little or nothing (other places inside the block measured the same).  LDS returns in order: when the block starts, the pairs of the next two blocks (four
    // reads) may still be on their way.
#define FXP_WTEXT(OFF0, OFF1, XPRE, XASM)                                                            \
    "s_waitcnt lgkmcnt(4)\n"                                                                         \
    "v_mfma_f32_16x16x32_bf16 %[a0], %[w0], %[c0], %[a0]\n"                                           \
    "ds_read_b128 %[n0], %[naddr] offset:" #OFF0 "\n"                                                 \
    "v_mfma_f32_16x16x32_bf16 %[a1], %[w1], %[c0], %[a1]\n"                                           \
    "ds_read_b128 %[n1], %[naddr] offset:" #OFF1 "\n"                                                 \
    "v_mfma_f32_16x16x32_bf16 %[a2], %[w2], %[c0], %[a2]\n"                                           \
    XPRE                                                                                             \
    "v_mfma_f32_16x16x32_bf16 %[a3], %[w3], %[c0], %[a3]\n"                                           \
    XASM                                                                                             \
    "v_mfma_f32_16x16x32_bf16 %[b0], %[w0], %[c1], %[b0]\n"                                           \
    "v_mfma_f32_16x16x32_bf16 %[b1], %[w1], %[c1], %[b1]\n"                                           \
    "v_mfma_f32_16x16x32_bf16 %[b2], %[w2], %[c1], %[b2]\n"                                           \
    "v_mfma_f32_16x16x32_bf16 %[b3], %[w3], %[c1], %[b3]\n"
#define FXP_WINS(W, NADDR, C0, C1)                                                                   \
    [naddr] "v"(NADDR), [w0] "v"(W[0]), [w1] "v"(W[1]), [w2] "v"(W[2]), [w3] "v"(W[3]), [c0] "v"(C0), [c1] "v"(C1)
    // block without a load
#define FXP_WBLOCK_N(W, N0, N1, NADDR, OFF0, OFF1, C0, C1, M)                                        \
    asm volatile(FXP_WTEXT(OFF0, OFF1, "", "")                                                           \
                 : [n0] "=&v"(N0), [n1] "=&v"(N1), FXP_ACC8(M) : FXP_WINS(W, NADDR, C0, C1) : "memory");
    // block that carries token-row DMA instruction I of the stage (M0 = LDS address of lane 0's 16 bytes)
#define FXP_WBLOCK_X(W, N0, N1, NADDR, OFF0, OFF1, C0, C1, M, I, XB, BUF)                            \
    asm volatile(FXP_WTEXT(OFF0, OFF1, "s_mov_b32 m0, %[ld]\n", "global_load_lds_dwordx4 %[xo], %[xb]\n") \
                 : [n0] "=&v"(N0), [n1] "=&v"(N1), FXP_ACC8(M)                                        \
                 : FXP_WINS(W, NADDR, C0, C1), [ld] "s"(lds_dma + (BUF) * kWdStageBytes + (I) * 1024), [xo] "v"(xoff[I]), [xb] "s"(XB) \
                 : "memory");
    // block that carries one weight load
#define FXP_WBLOCK_W(W, N0, N1, NADDR, OFF0, OFF1, C0, C1, M, WD, WB, WOFF)                          \
    asm volatile(FXP_WTEXT(OFF0, OFF1, "", "global_load_dwordx4 %[wd], %[wo], %[wb] offset:" #WOFF "\n")  \
                 : [n0] "=&v"(N0), [n1] "=&v"(N1), FXP_ACC8(M), [wd] "=&v"(WD)                        \
                 : FXP_WINS(W, NADDR, C0, C1), [wo] "v"(wlane), [wb] "s"(WB) : "memory");
    u32x4 x0a, x0b, x1a, x1b, x2a, x2b, x3a, x3b;          // four operand pairs: block j of a k-step multiplies pair j % 4
    // One k-step (16 column tiles, 64 MFMAs) in eight blocks, each carrying one load of the stage.  ADDR: this lane's slot
    // of column tile 0 of this k-step; NEXT: of the next one.
#define FXP_WKSTEP_X(W, ADDR, NEXT, XB, BUF)                                      \
    FXP_WBLOCK_X(W, x3a, x3b, ADDR, 12288, 14336, x0a, x0b, 0, 0, XB, BUF)        \
    FXP_WBLOCK_X(W, x0a, x0b, ADDR, 16384, 18432, x1a, x1b, 2, 1, XB, BUF)        \
    FXP_WBLOCK_X(W, x1a, x1b, ADDR, 20480, 22528, x2a, x2b, 4, 2, XB, BUF)        \
    FXP_WBLOCK_X(W, x2a, x2b, ADDR, 24576, 26624, x3a, x3b, 6, 3, XB, BUF)        \
    FXP_WBLOCK_X(W, x3a, x3b, ADDR, 28672, 30720, x0a, x0b, 8, 4, XB, BUF)        \
    FXP_WBLOCK_X(W, x0a, x0b, NEXT, 0, 2048, x1a, x1b, 10, 5, XB, BUF)            \
    FXP_WBLOCK_X(W, x1a, x1b, NEXT, 4096, 6144, x2a, x2b, 12, 6, XB, BUF)         \
    FXP_WBLOCK_X(W, x2a, x2b, NEXT, 8192, 10240, x3a, x3b, 14, 7, XB, BUF)
#define FXP_WKSTEP_W(W, ADDR, NEXT, WN, WB0, WB1)                                 \
    FXP_WBLOCK_W(W, x3a, x3b, ADDR, 12288, 14336, x0a, x0b, 0, WN[0][0], WB0, 0)    \
    FXP_WBLOCK_W(W, x0a, x0b, ADDR, 16384, 18432, x1a, x1b, 2, WN[0][1], WB0, 1024) \
    FXP_WBLOCK_W(W, x1a, x1b, ADDR, 20480, 22528, x2a, x2b, 4, WN[0][2], WB0, 2048) \
    FXP_WBLOCK_W(W, x2a, x2b, ADDR, 24576, 26624, x3a, x3b, 6, WN[0][3], WB0, 3072) \
    FXP_WBLOCK_W(W, x3a, x3b, ADDR, 28672, 30720, x0a, x0b, 8, WN[1][0], WB1, 0)    \
    FXP_WBLOCK_W(W, x0a, x0b, NEXT, 0, 2048, x1a, x1b, 10, WN[1][1], WB1, 1024)     \
    FXP_WBLOCK_W(W, x1a, x1b, NEXT, 4096, 6144, x2a, x2b, 12, WN[1][2], WB1, 2048)  \
    FXP_WBLOCK_W(W, x2a, x2b, NEXT, 8192, 10240, x3a, x3b, 14, WN[1][3], WB1, 3072)
#define FXP_WKSTEP_N(W, ADDR, NEXT)                                               \
    FXP_WBLOCK_N(W, x3a, x3b, ADDR, 12288, 14336, x0a, x0b, 0)                    \
    FXP_WBLOCK_N(W, x0a, x0b, ADDR, 16384, 18432, x1a, x1b, 2)                    \
    FXP_WBLOCK_N(W, x1a, x1b, ADDR, 20480, 22528, x2a, x2b, 4)                    \
    FXP_WBLOCK_N(W, x2a, x2b, ADDR, 24576, 26624, x3a, x3b, 6)                    \
    FXP_WBLOCK_N(W, x3a, x3b, ADDR, 28672, 30720, x0a, x0b, 8)                    \
    FXP_WBLOCK_N(W, x0a, x0b, NEXT, 0, 2048, x1a, x1b, 10)                        \
    FXP_WBLOCK_N(W, x1a, x1b, NEXT, 4096, 6144, x2a, x2b, 12)                     \
    FXP_WBLOCK_N(W, x2a, x2b, NEXT, 8192, 10240, x3a, x3b, 14)

    // ring of four stages of weights (two k-steps of four tiles each); W(s) lives in set s % 4
    u32x4 w[4][2][kWdRn];
    // prologue: token rows and weights of stages 0..2
#pragma unroll
    for (int st = 0; st < 3; ++st) {
        const char *xb = xptr(st);
#pragma unroll
        for (int i = 0; i < 8; ++i)
            asm volatile("s_mov_b32 m0, %[ld]\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %[xo], %[xb]\n"
                         : : [ld] "s"(lds_dma + st * kWdStageBytes + i * 1024), [xo] "v"(xoff[i]), [xb] "s"(xb) : "memory");
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int r = 0; r < kWdRn; ++r)       // (assembly, like every load of this kernel: the compiler must not count it)
                asm volatile("global_load_dwordx4 %[wd], %[wo], %[wb]" : [wd] "=&v"(w[st][h][r])
                             : [wo] "v"(wlane), [wb] "s"(wptr(2 * st + h) + r * 1024) : "memory");
    }
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    if constexpr (PROBE != 0) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int r = 0; r < kWdRn; ++r) w[3][h][r] = w[1][h][r];
    }
    asm volatile("ds_read_b128 %[p0], %[addr]\n"
                 "ds_read_b128 %[p1], %[addr] offset:2048\n"
                 "ds_read_b128 %[p2], %[addr] offset:4096\n"
                 "ds_read_b128 %[p3], %[addr] offset:6144\n"
                 "ds_read_b128 %[p4], %[addr] offset:8192\n"
                 "ds_read_b128 %[p5], %[addr] offset:10240\n"
                 : [p0] "=&v"(x0a), [p1] "=&v"(x0b), [p2] "=&v"(x1a), [p3] "=&v"(x1b), [p4] "=&v"(x2a), [p5] "=&v"(x2b)
                 : [addr] "v"(lds_h0) : "memory");

    // Stage s: multiply X(s) (buffer s % 4) by W(s); meanwhile ask for X(s+3) -> buffer (s+3) % 4 and W(s+3) -> set
    // (s+3) % 4 (both last used in stage s-1, behind the barrier that ended it).  The barrier at the end of the stage
    // publishes X(s+2) for the first operand reads of stage s+2, which the last blocks of stage s+1 issue, and W(s+1)
    // must have landed: the vector-memory counter is in order, so at that point W(s+2) (asked for a stage ago, behind
    // X(s+2)) and this stage's own sixteen loads may still be in flight: 24.
#define FXP_WSTAGE(S, KT0) {                                                                                 \
    const char *xb = xptr((KT0) + (S) + 3), *wb0 = wptr(2 * ((KT0) + (S) + 3)), *wb1 = wptr(2 * ((KT0) + (S) + 3) + 1); \
    if constexpr (PROBE == 0) {                                                                              \
        FXP_WKSTEP_X(w[(S) % 4][0], lds_h0 + ((S) % 4) * kWdStageBytes, lds_h1 + ((S) % 4) * kWdStageBytes, xb, ((S) + 3) % 4) \
        FXP_WKSTEP_W(w[(S) % 4][1], lds_h1 + ((S) % 4) * kWdStageBytes, lds_h0 + (((S) + 1) % 4) * kWdStageBytes, \
                     w[((S) + 3) % 4], wb0, wb1)                                                            \
        asm volatile("s_waitcnt vmcnt(24)\n\ts_barrier" ::: "memory");                                       \
    } else {                                                                                                 \
        FXP_WKSTEP_N(w[(S) % 4][0], lds_h0 + ((S) % 4) * kWdStageBytes, lds_h1 + ((S) % 4) * kWdStageBytes) \
        FXP_WKSTEP_N(w[(S) % 4][1], lds_h1 + ((S) % 4) * kWdStageBytes, lds_h0 + (((S) + 1) % 4) * kWdStageBytes) \
        asm volatile("s_barrier" ::: "memory");                                                              \
    } }
    for (int kt = 0; kt < KT; kt += 4) {
        FXP_WSTAGE(0, kt)
        FXP_WSTAGE(1, kt)
        FXP_WSTAGE(2, kt)
        FXP_WSTAGE(3, kt)
    }
    // loads past the end (clamped, never used) must have landed before their registers or LDS are given up
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" : "+v"(x0a), "+v"(x0b), "+v"(x1a), "+v"(x1b), "+v"(x2a), "+v"(x2b) : : "memory");
#undef FXP_WSTAGE
#undef FXP_WKSTEP_X
#undef FXP_WKSTEP_W
#undef FXP_WKSTEP_N
#undef FXP_WBLOCK_X
#undef FXP_WBLOCK_W
#undef FXP_WBLOCK_N
#undef FXP_WINS
#undef FXP_WTEXT
#undef FXP_ACC8

    // ---- epilogue (as above; lane holds 4 consecutive n of token row m0 + mt*16 + col)
    if constexpr (EPI == kEpiRope) {
        // q|k|v projection: the rotary embedding and the cache append happen here.  The row tiles of a q or k head
        // were packed with the halves of the head dimension alternating, so accumulator tiles (r, r+1) of this lane
        // hold the rotary pair (d, d + D/2) of one token; the wave's four tiles lie inside one head and one of the q,
        // k, v sections (sections and heads start at multiples of four tiles).
        const RopeArgs &ra = a.rope;
        const int D = ra.head_dim, tiles_per_head = D / 16, half = D / 2;
        const int q_tiles = ra.n_q_heads * tiles_per_head, kv_tiles = ra.n_kv_heads * tiles_per_head;
        const int sect = nt0 < q_tiles ? 0 : (nt0 < q_tiles + kv_tiles ? 1 : 2);            // q, k, v (wave-uniform)
        const int nts = nt0 - (sect == 0 ? 0 : sect == 1 ? q_tiles : q_tiles + kv_tiles);   // tile inside the section
        const int head = nts / tiles_per_head, j0 = nts % tiles_per_head;                  // j0: 0 or 4
        const int64_t Nq = (int64_t)ra.n_q_heads * D;
        // the cache row of each of this lane's tokens (all requests first, then the uses)
        int32_t trow[kWdRm];
        if (sect != 0) {
#pragma unroll
            for (int mt = 0; mt < kWdRm; ++mt) trow[mt] = ra.tok_row[min(m0 + mt * 16 + col, a.M - 1)];
        }
        // Every wait for a load also waits for the stores before it (one counter), and the compiler waits for a load right
        // where it is used: loads scattered between the stores made this epilogue a chain of round trips.  So the loads
        // come in batches ahead of the stores: the bias once, the cos / sin rows of four token tiles at a time.
        if (nt0 < a.NT) {
            u32x2 bias_v[kWdRn];
#pragma unroll
            for (int r = 0; r < kWdRn; ++r)
                bias_v[r] = a.bias ? *reinterpret_cast<const u32x2 *>(a.bias + (nt0 + r) * 16 + 4 * c) : u32x2{0u, 0u};
            auto rounded = [&](int r, int mt, float (&y)[4]) {     // the projection's values as bf16 (+ bias), as the unfused path stores them
                y[0] = acc[r][mt][0] + bf16_lo(bias_v[r].x); y[1] = acc[r][mt][1] + bf16_hi(bias_v[r].x);
                y[2] = acc[r][mt][2] + bf16_lo(bias_v[r].y); y[3] = acc[r][mt][3] + bf16_hi(bias_v[r].y);
                const uint32_t p0 = pack_bf16x2(y[0], y[1]), p1 = pack_bf16x2(y[2], y[3]);
                y[0] = bf16_lo(p0); y[1] = bf16_hi(p0); y[2] = bf16_lo(p1); y[3] = bf16_hi(p1);
            };
            constexpr int kGroup = 4;
#pragma unroll
            for (int mg = 0; mg < kWdRm; mg += kGroup) {
                f32x4_t co[kGroup][2], si[kGroup][2];
                if (sect != 2) {
#pragma unroll
                    for (int g = 0; g < kGroup; ++g)
#pragma unroll
                        for (int pr = 0; pr < 2; ++pr) {
                            const int64_t at = (int64_t)min(m0 + (mg + g) * 16 + col, a.M - 1) * half + ((j0 + 2 * pr) / 2) * 16 + 4 * c;
                            co[g][pr] = *reinterpret_cast<const f32x4_t *>(ra.cs + at);
                            si[g][pr] = *reinterpret_cast<const f32x4_t *>(ra.sn + at);
                        }
                }
#pragma unroll
                for (int g = 0; g < kGroup; ++g) {
                    const int mt = mg + g;
                    const int m = m0 + mt * 16 + col;
                    if (m >= a.M) continue;
                    // destination of dim 0 of this head for token m
                    uint16_t *dst;
                    if (sect == 0) dst = ra.q_out + (int64_t)m * Nq + (int64_t)head * D;
                    else dst = ra.pool + ((int64_t)ra.layer_local * ra.num_blocks * 2 * ra.n_kv_heads * kBlockTokens + trow[mt] +
                                          ((sect - 1) * ra.n_kv_heads + head) * kBlockTokens) * D;
                    if (sect == 2) {
                        // v rows: natural order, no rotation
#pragma unroll
                        for (int r = 0; r < kWdRn; ++r) {
                            float y[4];
                            rounded(r, mt, y);
                            *reinterpret_cast<u32x2 *>(dst + (j0 + r) * 16 + 4 * c) = u32x2{pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3])};
                        }
                    } else {
#pragma unroll
                        for (int pr = 0; pr < 2; ++pr) {
                            const int r = 2 * pr;
                            const int d = ((j0 + r) / 2) * 16 + 4 * c;          // dim of the first-half value; its partner is d + D/2
                            float lo[4], hi[4];
                            rounded(r, mt, lo);
                            rounded(r + 1, mt, hi);
                            float rl[4], rh[4];
#pragma unroll
                            for (int v = 0; v < 4; ++v) {
                                rl[v] = lo[v] * co[g][pr][v] - hi[v] * si[g][pr][v];
                                rh[v] = hi[v] * co[g][pr][v] + lo[v] * si[g][pr][v];
                            }
                            *reinterpret_cast<u32x2 *>(dst + d) = u32x2{pack_bf16x2(rl[0], rl[1]), pack_bf16x2(rl[2], rl[3])};
                            *reinterpret_cast<u32x2 *>(dst + d + half) = u32x2{pack_bf16x2(rh[0], rh[1]), pack_bf16x2(rh[2], rh[3])};
                        }
                    }
                }
            }
        }
        return;
    }
    // (loads in batches ahead of the stores, as in the rotary epilogue: the bias once, the residual -- which may be the
    // output buffer itself, so that no load can be moved across a store -- for four token tiles at a time; a lane reads
    // only the addresses it writes itself)
    u32x2 bias_v[kWdRn];
#pragma unroll
    for (int r = 0; r < kWdRn; ++r)
        bias_v[r] = (EPI != kEpiSwiglu && a.bias) ? *reinterpret_cast<const u32x2 *>(a.bias + min(nt0 + r, a.NT - 1) * 16 + 4 * c) : u32x2{0u, 0u};
    constexpr int kGroup = 4;
#pragma unroll
    for (int mg = 0; mg < kWdRm; mg += kGroup) {
        u32x2 resid[kGroup][kWdRn];
        if constexpr (EPI == kEpiResidual) {
#pragma unroll
            for (int g = 0; g < kGroup; ++g)
#pragma unroll
                for (int r = 0; r < kWdRn; ++r)
                    resid[g][r] = *reinterpret_cast<const u32x2 *>(a.R + (int64_t)min(m0 + (mg + g) * 16 + col, a.M - 1) * a.ldc +
                                                                   min(nt0 + r, a.NT - 1) * 16 + 4 * c);
        }
#pragma unroll
        for (int g = 0; g < kGroup; ++g) {
            const int mt = mg + g;
            const int m = m0 + mt * 16 + col;
            if (m >= a.M) continue;
            if constexpr (EPI == kEpiSwiglu) {
#pragma unroll
                for (int r = 0; r < kWdRn; r += 2) {
                    if (nt0 + r >= a.NT) continue;
                    const int f = ((nt0 + r) / 2) * 16 + 4 * c;
                    float y[4];
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const float gt = acc[r][mt][v];
                        y[v] = gt / (1.f + __expf(-gt)) * acc[r + 1][mt][v];
                    }
                    *reinterpret_cast<u32x2 *>(a.C + (int64_t)m * a.ldc + f) = u32x2{pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3])};
                }
            } else {
#pragma unroll
                for (int r = 0; r < kWdRn; ++r) {
                    if (nt0 + r >= a.NT) continue;
                    const int n = (nt0 + r) * 16 + 4 * c;
                    float y[4] = {acc[r][mt][0] + bf16_lo(bias_v[r].x), acc[r][mt][1] + bf16_hi(bias_v[r].x),
                                  acc[r][mt][2] + bf16_lo(bias_v[r].y), acc[r][mt][3] + bf16_hi(bias_v[r].y)};
                    if constexpr (EPI == kEpiRelu) {
#pragma unroll
                        for (int v = 0; v < 4; ++v) y[v] = fmaxf(y[v], 0.f);
                    }
                    if constexpr (EPI == kEpiResidual) {
                        const u32x2 rv = resid[g][r];
                        y[0] += bf16_lo(rv.x); y[1] += bf16_hi(rv.x); y[2] += bf16_lo(rv.y); y[3] += bf16_hi(rv.y);
                    }
                    *reinterpret_cast<u32x2 *>(a.C + (int64_t)m * a.ldc + n) = u32x2{pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3])};
                }
            }
        }
    }
}

// Which tile takes a launch.  The wide tile needs a shape that fits it; then the two are compared by a model of their
// running times in units of one 256 x 256 x K tile at the wide kernel's rate, fitted to measurements at 2048 .. 15,928
// rows of the 7B shape (it picks the faster kernel in every one of them):
//   wide: one workgroup per CU, so rounds = ceil(tiles / CUs), one unit each;
//   256 x 128: two workgroups per CU take 1.11 units per double round; a last round with at most one workgroup per CU
//         runs each of them alone in 0.68.
static bool wide_tile_fits(const TiledArgs &a)
{
    static const int off = tuning_int("FXP_NO_WIDE_TILE", 0), force_rows = tuning_int("FXP_WIDE_MIN_ROWS", 0);
    static const int no_rope = tuning_int("FXP_NO_ROPE_EPILOGUE", 0);
    if (a.epilogue == kEpiRope && (no_rope || a.rope.head_dim % 64 != 0 || (a.rope.n_q_heads + 2 * a.rope.n_kv_heads) * (a.rope.head_dim / 16) != a.NT))
        return false;
    if (off || a.epilogue == kEpiPartial || a.M < 4 * kWdBM || a.K % 256 != 0 || a.NT % kWdRn != 0 ||
        (int64_t)a.M * a.ldx * 2 >= (int64_t(1) << 32))
        return false;
    if (force_rows > 0) return a.M >= force_rows;
    const int cus = device_cus();
    const int64_t tiles_n = (a.NT * 16 + kWdBN - 1) / kWdBN;
    const int64_t wide_wgs = tiles_n * ((a.M + kWdBM - 1) / kWdBM), narrow_wgs = tiles_n * ((a.M + kTgBM - 1) / kTgBM);
    const double t_wide = (double)((wide_wgs + cus - 1) / cus);
    const int64_t pairs = narrow_wgs / (2 * cus), rest = narrow_wgs - pairs * 2 * cus;
    const double t_narrow = 1.11 * (double)pairs + (rest == 0 ? 0.0 : rest <= cus ? 0.68 : 1.11);
    return t_wide < t_narrow;
}

bool gemm_wide_applies(const TiledArgs &a) { return wide_tile_fits(a); }

template <int EPI, int PROBE>
static hipError_t launch_wide_probe(const TiledArgs &a_in, hipStream_t stream)
{
    // allow 128 KiB of dynamic LDS: once per kernel instantiation and device
    static bool lds_set[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (!lds_set[dev]) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_wide_kernel<EPI, PROBE>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kWdLdsBytes);
        if (e != hipSuccess) return e;
        lds_set[dev] = true;
    }
    const int tiles_n = (a_in.NT * 16 + kWdBN - 1) / kWdBN, tiles_m = (a_in.M + kWdBM - 1) / kWdBM;
    TiledArgs a = a_in;
    int blocks = 0;
    for (int bm = 8; bm >= 1; bm /= 2) {           // super-block shape with the fewest padded slots (ties: the squarer one)
        const int bn = 32 / bm, padded = ((tiles_n + bn - 1) / bn) * ((tiles_m + bm - 1) / bm);
        if (blocks == 0 || padded < blocks) { blocks = padded; a.blk_m = bm; }
    }
    const dim3 grid((blocks + kXcds - 1) / kXcds * kXcds * 32);
    hipLaunchKernelGGL((gemm_wide_kernel<EPI, PROBE>), grid, dim3(kTgThreads), kWdLdsBytes, stream, a);
    return hipGetLastError();
}

template <int EPI>
static hipError_t launch_wide(const TiledArgs &a, hipStream_t stream)
{
#ifdef FXP_TUNING
    static const int probe = tuning_int("FXP_WIDE_PROBE", 0);
    if (probe) return launch_wide_probe<EPI, 1>(a, stream);
#endif
    return launch_wide_probe<EPI, 0>(a, stream);
}

hipError_t launch_gemm_tiled(const TiledArgs &a, hipStream_t stream)
{
    if (wide_tile_fits(a)) {
        switch (a.epilogue) {
        case kEpiStore: return launch_wide<kEpiStore>(a, stream);
        case kEpiResidual: return launch_wide<kEpiResidual>(a, stream);
        case kEpiSwiglu: return launch_wide<kEpiSwiglu>(a, stream);
        case kEpiRelu: return launch_wide<kEpiRelu>(a, stream);
        case kEpiRope: return launch_wide<kEpiRope>(a, stream);
        default: break;
        }
    }
    if (a.epilogue == kEpiRope) return hipErrorInvalidValue;       // only the wide tile finishes q|k|v itself
    const int tiles_n = (a.NT * 16 + kTgBN - 1) / kTgBN;
    const int tiles_m = (a.M + kTgBM - 1) / kTgBM;
    // the XCD-aware numbering covers whole 4 x 8 super-blocks, rounded up to a multiple of 8 of them
    const int blocks = ((tiles_n + 3) / 4) * ((tiles_m + 7) / 8);
    dim3 grid((blocks + kXcds - 1) / kXcds * kXcds * 32, a.epilogue == kEpiPartial ? a.S : 1);
    if (tiles_m == 1) grid.x = tiles_n;
    else if (tiles_m < 16) grid.x = (tiles_n + kXcds - 1) / kXcds * kXcds * tiles_m;
    const bool tail = a.K % 64 != 0;                  // a stage is 64 wide: the token rows end inside the last one
    static const int early_tiles = tuning_int("FXP_TILED_EARLY_W_TILES", 2);
    const bool early = tiles_m <= early_tiles;        // few row tiles: bound by the weight stream, see the kernel
#define FXP_TG_LAUNCH(E)                                                                                       \
    if (tail) {                                                                                                \
        if (early) hipLaunchKernelGGL((gemm_tiled_kernel<E, true, true>), grid, dim3(kTgThreads), 0, stream, a);   \
        else hipLaunchKernelGGL((gemm_tiled_kernel<E, true, false>), grid, dim3(kTgThreads), 0, stream, a);    \
    } else {                                                                                                   \
        if (early) hipLaunchKernelGGL((gemm_tiled_kernel<E, false, true>), grid, dim3(kTgThreads), 0, stream, a);  \
        else hipLaunchKernelGGL((gemm_tiled_kernel<E, false, false>), grid, dim3(kTgThreads), 0, stream, a);   \
    }
    switch (a.epilogue) {
    case kEpiStore: FXP_TG_LAUNCH(kEpiStore) break;
    case kEpiResidual: FXP_TG_LAUNCH(kEpiResidual) break;
    case kEpiSwiglu: FXP_TG_LAUNCH(kEpiSwiglu) break;
    case kEpiPartial: FXP_TG_LAUNCH(kEpiPartial) break;
    case kEpiRelu: FXP_TG_LAUNCH(kEpiRelu) break;
    default: return hipErrorInvalidValue;
    }
#undef FXP_TG_LAUNCH
    return hipGetLastError();
}

}  // namespace fxp
