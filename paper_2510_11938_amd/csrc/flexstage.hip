// C ABI of the library (include/flexstage.h): argument validation, the stage
// handle, workspace carving and the per-layer launch sequence.  All arithmetic
// is in the kernels; this file only decides which kernel runs on which buffer.
#include "../../include/flexstage.h"
#include "kernels.h"

#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <algorithm>
#include <mutex>
#include <new>

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int hip_fail(hipError_t e, const char *what)
{
    return fail(FXP_EHIP, "%s: %s", what, hipGetErrorString(e));
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int k_steps(int K) { return (K + 63) / 64 * 2; }                   // 32-wide steps, K padded to 64
inline size_t packed_bytes(int N, int K) { return (size_t)((N / 16 + fxp::kPackGroup - 1) / fxp::kPackGroup * fxp::kPackGroup) * k_steps(K) * 1024; }   // whole groups of tiles

constexpr int kSkinnyMaxTokens = 128;     // up to here the projections run weight-streaming with split-K
constexpr int kSkinnyWideTokens = 64;     // above this the split-K work goes to the tiled kernel's 128-row tile

int check_desc(const fxp_stage_desc *d)
{
    if (!d) return fail(FXP_EINVAL, "stage descriptor is null");
    if (d->layer_begin < 0 || d->layer_end <= d->layer_begin) return fail(FXP_EINVAL, "bad layer range [%d,%d)", d->layer_begin, d->layer_end);
    if (d->kv_block_size != 16) return fail(FXP_EINVAL, "kv_block_size must be 16 (got %d)", d->kv_block_size);
    if (d->head_dim != 64 && d->head_dim != 128) return fail(FXP_EINVAL, "head_dim must be 64 or 128 (got %d)", d->head_dim);
    if (d->n_kv_heads <= 0 || d->n_q_heads <= 0 || d->n_q_heads % d->n_kv_heads)
        return fail(FXP_EINVAL, "n_q_heads (%d) must be a positive multiple of n_kv_heads (%d)", d->n_q_heads, d->n_kv_heads);
    if (!fxp::decode_attn_supported(d->head_dim, d->n_q_heads / d->n_kv_heads))
        return fail(FXP_EINVAL, "query heads per kv head must be 1..16 (got %d)", d->n_q_heads / d->n_kv_heads);
    if (d->hidden <= 0 || d->hidden % 16 || d->ffn <= 0 || d->ffn % 16)
        return fail(FXP_EINVAL, "hidden (%d) and ffn (%d) must be positive multiples of 16", d->hidden, d->ffn);
    if (d->arch != FXP_ARCH_LLAMA && d->arch != FXP_ARCH_OPT) return fail(FXP_EINVAL, "unknown layer kind %d", d->arch);
    if (!(d->rms_eps >= 0.f) || (d->arch == FXP_ARCH_LLAMA && !(d->rope_base > 1.f))) return fail(FXP_EINVAL, "bad rms_eps or rope_base");
    return FXP_OK;
}

// KV geometry checks shared by the repartition calls (only these fields are read)
int check_kv_geom(const fxp_stage_desc *d)
{
    if (!d) return fail(FXP_EINVAL, "stage descriptor is null");
    if (d->kv_block_size != 16) return fail(FXP_EINVAL, "kv_block_size must be 16 (got %d)", d->kv_block_size);
    if (d->n_kv_heads <= 0 || d->head_dim <= 0 || d->head_dim % 8)
        return fail(FXP_EINVAL, "bad kv geometry: n_kv_heads %d head_dim %d", d->n_kv_heads, d->head_dim);
    return FXP_OK;
}

struct LayerRecord {           // offsets into one layer's contiguous record in the arena
    size_t wqkv, wo, wgu, wd, g_attn, g_ffn, bytes;
    size_t b_attn, b_ffn, b_qkv, b_o, b_up, b_down;     // OPT-style layers only
};

LayerRecord layer_record(const fxp_stage_desc &d)
{
    LayerRecord r;
    const int Nqkv = (d.n_q_heads + 2 * d.n_kv_heads) * d.head_dim, Nq = d.n_q_heads * d.head_dim;
    size_t at = 0;
    r.wqkv = at; at += align_up(packed_bytes(Nqkv, d.hidden), 256);
    r.wo = at;   at += align_up(packed_bytes(d.hidden, Nq), 256);
    const bool opt = d.arch == FXP_ARCH_OPT;
    r.wgu = at;  at += align_up(packed_bytes((opt ? 1 : 2) * d.ffn, d.hidden), 256);     // gate|up interleaved, or the first feed-forward matrix
    r.wd = at;   at += align_up(packed_bytes(d.hidden, d.ffn), 256);
    r.g_attn = at; at += align_up((size_t)d.hidden * 2, 256);
    r.g_ffn = at;  at += align_up((size_t)d.hidden * 2, 256);
    r.b_attn = r.b_ffn = r.b_qkv = r.b_o = r.b_up = r.b_down = 0;
    if (opt) {
        r.b_attn = at; at += align_up((size_t)d.hidden * 2, 256);
        r.b_ffn = at;  at += align_up((size_t)d.hidden * 2, 256);
        r.b_qkv = at;  at += align_up((size_t)Nqkv * 2, 256);
        r.b_o = at;    at += align_up((size_t)d.hidden * 2, 256);
        r.b_up = at;   at += align_up((size_t)d.ffn * 2, 256);
        r.b_down = at; at += align_up((size_t)d.hidden * 2, 256);
    }
    r.bytes = at;
    return r;
}

using fxp::device_cus;
int env_int(const char *name, int dflt) { return fxp::tuning_int(name, dflt); }

// Launch shape of a skinny projection: R weight tiles per wavefront (workgroup =
// 4 wavefronts = 64*R rows) and the split-K factor S.  Enough workgroups to put
// several wavefronts on every CU, but as few splits as that allows: every split
// adds a float slice of partial sums that the epilogue has to read back.
// Depends on shapes only, so results do not depend on anything else.
struct SkinnyCfg { int R, S; };
// The gate|up projection applies SwiGLU in its epilogue (no split-K, no partial sums) when its
// 2F weight rows alone give every second CU a workgroup (128 rows each) or more.
bool skinny_fused_swiglu(int N2)
{
    static const int off = env_int("FXP_NO_FUSED_SWIGLU", 0);
    return !off && N2 / 128 >= device_cus() / 2;
}

SkinnyCfg skinny_cfg(int N, int K, int M)
{
    static const int forced_s = env_int("FXP_SKINNY_SPLIT", 0), forced_r = env_int("FXP_SKINNY_R", 0);
    static const int max_wgs = env_int("FXP_SKINNY_MAX_WGS", device_cus());
    const int ks = k_steps(K);
    SkinnyCfg c;
    // Measured on MI355X: about one workgroup (4 wavefronts, 8-16 KiB of weights in flight each)
    // per CU streams fastest; more, thinner workgroups lose bandwidth.
    c.R = forced_r ? forced_r : ((N >= 16384 && M <= 64) ? 4 : 2);
    if (M > kSkinnyWideTokens) {
        // above 64 rows the tiled kernel is used, whose workgroup covers 256 weight rows x 128 token rows: one
        // workgroup per CU of a 256-CU chip and never more (a second one on a quarter of the CUs doubles the
        // time of the launch; measured: 320 workgroups 57 us, 240 workgroups 45 us).  With several hundred
        // token rows a narrow matrix still has few tiles (hidden 4096: 16 x rows/128) and is split as well.
        const int wgs = ((N + 255) / 256) * ((M + 127) / 128);
        // Up to 16 pieces: a narrow matrix at 65..128 rows (hidden 4096 or 5120: 16 or 20 tiles) otherwise fills half
        // the chip, which costs more than the extra partial sums (7B shape, 128 rows: 130 -> 123 us per layer).
        static const int cap = env_int("FXP_TILED_SPLIT_CAP", 16);
        c.S = forced_s ? forced_s : std::max(1, std::min(std::min(cap, ks / 8), device_cus() / wgs));
        return c;
    }
    const int wgs_n = (N + 64 * c.R - 1) / (64 * c.R);
    int s = 1;
    if (M > 32) {
        // 33..64 rows: one workgroup per CU as well, with the ring of four register buffers (two workgroups per CU
        // with two buffers each had been the better of the two-buffer forms; with four buffers one per CU wins on
        // every shape tried: 7B 64 rows 117 -> 106 us per layer, 13B 143 -> 135, 70B 313 -> 305)
        static const int wgs64 = env_int("FXP_SKINNY_MAX_WGS64", device_cus()), cap64 = env_int("FXP_SKINNY_CAP64", 12);
        s = std::max(1, std::min(std::min(cap64, ks / 16), wgs64 / wgs_n));
    } else {
        // up to 32 rows: as many workgroups as fit once on a 256-CU chip, any integer split (13B and 70B shapes:
        // 320 workgroups 17.5 / 36 us, 240 workgroups 13.9 / 29 us for o / q|k|v)
        s = std::max(1, std::min(std::min(8, ks / 8), max_wgs / wgs_n));
        // a narrow matrix that would need the full eight splits to fill the chip (output width 4096: 32 x 8 workgroups)
        // fills it with one tile per wavefront and four splits as well (64 x 4), and half the partial sums to write
        // and to read back are worth more than the wider workgroup: 7B shape, o 11.9 -> 11.1 us, down 21.1 -> 19.7 us
        if (!forced_r && !forced_s && c.R == 2 && s == 8 && wgs_n * 8 <= max_wgs && ks / 4 >= 8) {
            c.R = 1;
            s = 4;
        }
    }
    c.S = forced_s ? forced_s : s;
    return c;
}
int choose_split(int N, int K, int M) { return skinny_cfg(N, K, M).S; }

// ---- optional per-kernel timing (fxp_profile_*): HIP events recorded on the caller's stream
enum KernelClass { kKcRmsnorm, kKcSkinny, kKcTiled, kKcRope, kKcAttnDecode, kKcAttnCombine, kKcAttnPrefill,
                   kKcResidNorm, kKcSwiglu, kKcKvMove, kKcRopeTable, kKcCount };
const char *const kKernelClassNames[kKcCount] = {"rmsnorm", "gemm_skinny", "gemm_tiled", "rope_kvwrite", "attn_decode",
                                                 "attn_decode_combine", "attn_prefill", "resid_norm", "swiglu", "kv_move",
                                                 "rope_table"};
struct Profiler {
    static constexpr int kMaxPairs = 8192;
    bool on = false;
    int used = 0, created = 0;
    hipEvent_t ev[kMaxPairs][2];
    int cls[kMaxPairs];
} g_prof;

struct KernelTimer {     // records an event pair around the launches made during its lifetime
    int slot = -1;
    hipStream_t st;
    KernelTimer(int kc, hipStream_t stream) : st(stream)
    {
        if (!g_prof.on || g_prof.used >= Profiler::kMaxPairs) return;
        if (g_prof.used >= g_prof.created) {
            if (hipEventCreate(&g_prof.ev[g_prof.created][0]) != hipSuccess) return;
            if (hipEventCreate(&g_prof.ev[g_prof.created][1]) != hipSuccess) return;
            ++g_prof.created;
        }
        slot = g_prof.used++;
        g_prof.cls[slot] = kc;
        (void)hipEventRecord(g_prof.ev[slot][0], st);
    }
    ~KernelTimer() { if (slot >= 0) (void)hipEventRecord(g_prof.ev[slot][1], st); }
};

}  // namespace

namespace fxp {
// error reporting for the host-only translation units of the library
int ctl_fail(int code, const char *msg) { return fail(code, "%s", msg); }

int device_cus()
{
    static int cus = 0;
    if (!cus) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess) cus = n;
        if (cus <= 0) cus = 256;          // no device visible (host-only use of the size queries): the MI355X count
    }
    return cus;
}
}

struct fxp_stage {
    fxp_stage_desc d;
    int n_layers;
    char *arena;
    LayerRecord rec;
};

namespace {

struct Workspace {
    uint16_t *x[2], *n, *q, *qkv, *o, *h, *a;
    float *P, *part_acc, *part_ml, *pf_acc, *pf_ml, *dbg_ml, *rope_cs, *rope_sn;
    int32_t *tok_seq, *tok_pos, *tok_row;
    int32_t *blk_prefix;    // decode attention: cache blocks (per head) before each sequence, [B + 1]
    int n_workers;
    size_t bytes;
};

Workspace carve(const fxp_stage_desc &d, int T, int B, int max_blocks, char *base)
{
    Workspace w;
    size_t at = 0;
    auto take = [&](size_t bytes) { char *p = base ? base + at : nullptr; at += align_up(bytes, 256); return p; };
    const int H = d.hidden, Nq = d.n_q_heads * d.head_dim, Nall = (d.n_q_heads + 2 * d.n_kv_heads) * d.head_dim, F = d.ffn;
    const size_t t = (size_t)(T > 0 ? T : 1);
    w.x[0] = (uint16_t *)take(t * H * 2);
    w.x[1] = (uint16_t *)take(t * H * 2);
    w.n = (uint16_t *)take(t * H * 2);
    w.h = (uint16_t *)take(t * H * 2);
    w.q = (uint16_t *)take(t * Nq * 2);
    w.o = (uint16_t *)take(t * Nq * 2);
    w.a = (uint16_t *)take(t * F * 2);
    w.qkv = (uint16_t *)take(T > kSkinnyMaxTokens ? t * Nall * 2 : 0);
    size_t pmax = 0;
    const int shapes[4][2] = {{Nall, H}, {H, Nq}, {2 * F, H}, {H, F}};
    for (auto &s : shapes) {
        // sized for every batch of up to T rows, so that a workspace for max_tokens serves smaller calls too: the split
        // factor is chosen per class of row counts (<= 32, <= 64, then per 128-row tile until the matrix alone fills the chip)
        auto need = [&](int m) {
            m = std::min(m, T > 0 ? T : 1);
            const size_t b = (size_t)choose_split(s[0], s[1], m) * m * s[0] * 4;
            if (b > pmax) pmax = b;
        };
        need(32);
        need(kSkinnyWideTokens);
        for (int tm = 1; tm <= 256; ++tm) {
            need(tm * 128);
            if (tm * 128 >= T || choose_split(s[0], s[1], tm * 128) == 1) break;
        }
    }
    w.P = (float *)take(pmax);
    (void)max_blocks;
    // wavefronts of the decode attention kernel per CU: eight, but four for the grouped-query kernel at head_dim 128,
    // whose wavefronts each keep twice the bytes in flight (70B shape, batch 128: 373 -> 360 us per layer)
    const int per_cu = (d.n_q_heads != d.n_kv_heads && d.head_dim == 128) ? fxp::kDecodeWorkersPerCu / 2 : fxp::kDecodeWorkersPerCu;
    w.n_workers = device_cus() * env_int("FXP_DECODE_WORKERS_PER_CU", per_cu) / 4 * 4;
    const size_t rows = ((size_t)w.n_workers + (size_t)(B > 0 ? B : 1) * d.n_kv_heads) * (d.n_q_heads / d.n_kv_heads);
    w.part_acc = (float *)take(rows * d.head_dim * 4);
    w.part_ml = (float *)take(rows * 2 * 4);
    const size_t pf_rows = fxp::prefill_piece_rows(d.n_q_heads, T);
    w.pf_acc = (float *)take(pf_rows * d.head_dim * 4);
    w.pf_ml = (float *)take(pf_rows * 2 * 4);
    w.dbg_ml = (float *)take(t * d.n_q_heads * 3 * 4);
    w.rope_cs = (float *)take(t * (d.head_dim / 2) * 4);
    w.rope_sn = (float *)take(t * (d.head_dim / 2) * 4);
    w.tok_seq = (int32_t *)take(t * 4);
    w.tok_pos = (int32_t *)take(t * 4);
    w.tok_row = (int32_t *)take(t * 4);
    w.blk_prefix = (int32_t *)take(((size_t)B + 1) * 4);
    w.bytes = at;
    return w;
}

}  // namespace

extern "C" {

const char *fxp_last_error(void) { return g_err; }
const char *fxp_version(void) { return "flexstage 0.1 (gfx950)"; }

int fxp_profile_enable(int on)
{
    g_prof.on = on != 0;
    g_prof.used = 0;
    return FXP_OK;
}

int fxp_profile_num_classes(void) { return kKcCount; }

const char *fxp_profile_class_name(int kernel_class)
{
    return (kernel_class >= 0 && kernel_class < kKcCount) ? kKernelClassNames[kernel_class] : nullptr;
}

int fxp_profile_read_launch(int index, int *kernel_class, double *ms)
{
    if (index < 0 || index >= g_prof.used || !kernel_class || !ms) return fail(FXP_EINVAL, "launch index %d out of range [0,%d)", index, g_prof.used);
    hipError_t e = hipEventSynchronize(g_prof.ev[index][1]);
    if (e != hipSuccess) return hip_fail(e, "hipEventSynchronize");
    float t = 0.f;
    if ((e = hipEventElapsedTime(&t, g_prof.ev[index][0], g_prof.ev[index][1])) != hipSuccess) return hip_fail(e, "hipEventElapsedTime");
    *kernel_class = g_prof.cls[index];
    *ms = t;
    return FXP_OK;
}

int fxp_profile_read(int kernel_class, double *total_ms, int64_t *launches)
{
    if (kernel_class < 0 || kernel_class >= kKcCount || !total_ms || !launches) return fail(FXP_EINVAL, "bad argument to fxp_profile_read");
    double sum = 0.0;
    int64_t n = 0;
    for (int i = 0; i < g_prof.used; ++i) {
        if (g_prof.cls[i] != kernel_class) continue;
        hipError_t e = hipEventSynchronize(g_prof.ev[i][1]);
        if (e != hipSuccess) return hip_fail(e, "hipEventSynchronize");
        float ms = 0.f;
        if ((e = hipEventElapsedTime(&ms, g_prof.ev[i][0], g_prof.ev[i][1])) != hipSuccess) return hip_fail(e, "hipEventElapsedTime");
        sum += ms; ++n;
    }
    *total_ms = sum; *launches = n;
    return FXP_OK;
}

size_t fxp_stage_weight_arena_bytes(const fxp_stage_desc *desc)
{
    if (check_desc(desc) != FXP_OK) return 0;
    return layer_record(*desc).bytes * (size_t)(desc->layer_end - desc->layer_begin);
}

int fxp_stage_create(const fxp_stage_desc *desc, const fxp_layer_weights *layers, void *weight_arena,
                     size_t weight_arena_bytes, void *hip_stream, fxp_stage **out)
{
    if (int rc = check_desc(desc)) return rc;
    if (!layers || !weight_arena || !out) return fail(FXP_EINVAL, "null argument to fxp_stage_create");
    if ((uintptr_t)weight_arena % 256) return fail(FXP_EINVAL, "weight arena must be 256-byte aligned");
    const fxp_stage_desc &d = *desc;
    const int L = d.layer_end - d.layer_begin;
    const LayerRecord rec = layer_record(d);
    if (weight_arena_bytes < rec.bytes * (size_t)L)
        return fail(FXP_ENOSPC, "weight arena too small: %zu < %zu", weight_arena_bytes, rec.bytes * (size_t)L);
    hipStream_t st = (hipStream_t)hip_stream;
    const int H = d.hidden, D = d.head_dim, Nq = d.n_q_heads * D, Nkv = d.n_kv_heads * D, F = d.ffn;
    for (int l = 0; l < L; ++l) {
        const fxp_layer_weights &w = layers[l];
        const bool opt = d.arch == FXP_ARCH_OPT;
        if (!w.g_attn || !w.wq || !w.wk || !w.wv || !w.wo || !w.g_ffn || (!opt && !w.w_gate) || !w.w_up || !w.w_down)
            return fail(FXP_EINVAL, "layer %d has a null weight pointer", d.layer_begin + l);
        if (opt && (w.w_gate || !w.b_attn_norm || !w.b_ffn_norm || !w.bq || !w.bk || !w.bv || !w.bo || !w.b_up || !w.b_down))
            return fail(FXP_EINVAL, "layer %d: an OPT-style layer has no gate matrix and needs every bias", d.layer_begin + l);
        char *base = (char *)weight_arena + rec.bytes * (size_t)l;
        hipError_t e;
        // q | k | v rows concatenated
        if ((e = fxp::launch_weight_pack(w.wq, Nq, H, base + rec.wqkv, k_steps(H), 0, 1, D / 32, st))) return hip_fail(e, "pack wq");
        if ((e = fxp::launch_weight_pack(w.wk, Nkv, H, base + rec.wqkv, k_steps(H), Nq / 16, 1, D / 32, st))) return hip_fail(e, "pack wk");
        if ((e = fxp::launch_weight_pack(w.wv, Nkv, H, base + rec.wqkv, k_steps(H), (Nq + Nkv) / 16, 1, 0, st))) return hip_fail(e, "pack wv");
        if ((e = fxp::launch_weight_pack(w.wo, H, Nq, base + rec.wo, k_steps(Nq), 0, 1, 0, st))) return hip_fail(e, "pack wo");
        if (opt) {
            if ((e = fxp::launch_weight_pack(w.w_up, F, H, base + rec.wgu, k_steps(H), 0, 1, 0, st))) return hip_fail(e, "pack w_up");
            // the q and k biases follow the tile order of their matrices' rows
            if ((e = fxp::launch_bias_pack(w.bq, Nq, base + rec.b_qkv, D / 32, st))) return hip_fail(e, "pack bq");
            if ((e = fxp::launch_bias_pack(w.bk, Nkv, base + rec.b_qkv + (size_t)Nq * 2, D / 32, st))) return hip_fail(e, "pack bk");
            const struct { const void *src; size_t off, n; } vecs[] = {
                {w.b_attn_norm, rec.b_attn, (size_t)H}, {w.b_ffn_norm, rec.b_ffn, (size_t)H},
                {w.bv, rec.b_qkv + (size_t)(Nq + Nkv) * 2, (size_t)Nkv},
                {w.bo, rec.b_o, (size_t)H}, {w.b_up, rec.b_up, (size_t)F}, {w.b_down, rec.b_down, (size_t)H}};
            for (const auto &v : vecs)
                if ((e = hipMemcpyAsync(base + v.off, v.src, v.n * 2, hipMemcpyDeviceToDevice, st))) return hip_fail(e, "copy bias");
        } else {
            // gate and up rows interleaved in 16-row tiles
            if ((e = fxp::launch_weight_pack(w.w_gate, F, H, base + rec.wgu, k_steps(H), 0, 2, 0, st))) return hip_fail(e, "pack w_gate");
            if ((e = fxp::launch_weight_pack(w.w_up, F, H, base + rec.wgu, k_steps(H), 1, 2, 0, st))) return hip_fail(e, "pack w_up");
        }
        if ((e = fxp::launch_weight_pack(w.w_down, H, F, base + rec.wd, k_steps(F), 0, 1, 0, st))) return hip_fail(e, "pack w_down");
        if ((e = hipMemcpyAsync(base + rec.g_attn, w.g_attn, (size_t)H * 2, hipMemcpyDeviceToDevice, st))) return hip_fail(e, "copy g_attn");
        if ((e = hipMemcpyAsync(base + rec.g_ffn, w.g_ffn, (size_t)H * 2, hipMemcpyDeviceToDevice, st))) return hip_fail(e, "copy g_ffn");
    }
    fxp_stage *s = new (std::nothrow) fxp_stage;
    if (!s) return fail(FXP_ENOSPC, "out of host memory");
    s->d = d; s->n_layers = L; s->arena = (char *)weight_arena; s->rec = rec;
    *out = s;
    return FXP_OK;
}

int fxp_stage_destroy(fxp_stage *stage)
{
    delete stage;
    return FXP_OK;
}

int fxp_stage_layers(const fxp_stage *stage, int32_t *layer_begin, int32_t *layer_end)
{
    if (!stage || !layer_begin || !layer_end) return fail(FXP_EINVAL, "null argument to fxp_stage_layers");
    *layer_begin = stage->d.layer_begin; *layer_end = stage->d.layer_end;
    return FXP_OK;
}

// Refinement / consolidation of stages on handles.  Every layer is one contiguous record of the
// arena, so a stage over a sub-range is the same arena seen from another record on: no weight is
// moved, re-tiled or copied, and no kernel runs.
int fxp_stage_split(const fxp_stage *stage, int32_t layer_mid, fxp_stage **lower, fxp_stage **upper)
{
    if (!stage || !lower || !upper) return fail(FXP_EINVAL, "null argument to fxp_stage_split");
    if (layer_mid <= stage->d.layer_begin || layer_mid >= stage->d.layer_end)
        return fail(FXP_EINVAL, "split point %d is not inside (%d,%d)", layer_mid, stage->d.layer_begin, stage->d.layer_end);
    fxp_stage *lo = new (std::nothrow) fxp_stage(*stage), *hi = new (std::nothrow) fxp_stage(*stage);
    if (!lo || !hi) { delete lo; delete hi; return fail(FXP_ENOSPC, "out of host memory"); }
    lo->d.layer_end = layer_mid; lo->n_layers = layer_mid - stage->d.layer_begin;
    hi->d.layer_begin = layer_mid; hi->n_layers = stage->d.layer_end - layer_mid;
    hi->arena = stage->arena + stage->rec.bytes * (size_t)lo->n_layers;
    *lower = lo; *upper = hi;
    return FXP_OK;
}

int fxp_stage_merge(const fxp_stage *lower, const fxp_stage *upper, fxp_stage **out)
{
    if (!lower || !upper || !out) return fail(FXP_EINVAL, "null argument to fxp_stage_merge");
    const fxp_stage_desc &a = lower->d, &b = upper->d;
    if (a.layer_end != b.layer_begin) return fail(FXP_EINVAL, "stages [%d,%d) and [%d,%d) are not adjacent", a.layer_begin, a.layer_end, b.layer_begin, b.layer_end);
    if (a.hidden != b.hidden || a.n_q_heads != b.n_q_heads || a.n_kv_heads != b.n_kv_heads || a.head_dim != b.head_dim ||
        a.ffn != b.ffn || a.arch != b.arch || a.rms_eps != b.rms_eps || a.rope_base != b.rope_base || a.kv_block_size != b.kv_block_size)
        return fail(FXP_EINVAL, "stages differ in model geometry");
    if (upper->arena != lower->arena + lower->rec.bytes * (size_t)lower->n_layers)
        return fail(FXP_EINVAL, "the upper stage's layer records do not follow the lower stage's in memory; "
                                "create the merged stage with fxp_stage_create instead");
    fxp_stage *m = new (std::nothrow) fxp_stage(*lower);
    if (!m) return fail(FXP_ENOSPC, "out of host memory");
    m->d.layer_end = b.layer_end; m->n_layers = lower->n_layers + upper->n_layers;
    *out = m;
    return FXP_OK;
}

size_t fxp_stage_workspace_bytes(const fxp_stage *stage, int32_t max_tokens, int32_t max_seqs, int32_t max_blocks_per_seq)
{
    if (!stage || max_tokens < 0 || max_seqs < 0 || max_blocks_per_seq < 0) { fail(FXP_EINVAL, "bad argument to fxp_stage_workspace_bytes"); return 0; }
    return carve(stage->d, max_tokens, max_seqs, max_blocks_per_seq, nullptr).bytes;
}

static int forward_impl(fxp_stage *stage, const fxp_kv_pool *pool, const fxp_batch *batch, const void *hidden_in,
                        void *hidden_out, void *workspace, size_t workspace_bytes, float *probs, int64_t probs_stride,
                        void *hip_stream)
{
    if (!stage || !pool || !batch) return fail(FXP_EINVAL, "null argument to fxp_stage_forward");
    const fxp_stage_desc &d = stage->d;
    const int T = batch->num_tokens, B = batch->num_seqs;
    if (T < 0 || B < 0) return fail(FXP_EINVAL, "negative batch size");
    if (B > FXP_MAX_SEQS) return fail(FXP_EINVAL, "num_seqs %d above the limit of %d", B, FXP_MAX_SEQS);
    if (T == 0 || B == 0) return FXP_OK;
    if (!hidden_in || !hidden_out || !workspace) return fail(FXP_EINVAL, "null buffer passed to fxp_stage_forward");
    if (!batch->cu_seqlens_q || !batch->ctx_lens || !batch->block_table) return fail(FXP_EINVAL, "null batch table");
    if (!pool->base || pool->num_blocks <= 0) return fail(FXP_EINVAL, "empty kv pool");
    if (pool->layer_begin != d.layer_begin || pool->layer_end != d.layer_end)
        return fail(FXP_EINVAL, "pool holds layers [%d,%d) but the stage is [%d,%d)", pool->layer_begin, pool->layer_end, d.layer_begin, d.layer_end);
    if (batch->max_q_len < 1 || batch->max_q_len > T) return fail(FXP_EINVAL, "max_q_len %d out of range for %d tokens", batch->max_q_len, T);
    if (batch->max_blocks_per_seq < 1) return fail(FXP_EINVAL, "max_blocks_per_seq must be positive");
    if ((uintptr_t)workspace % 256) return fail(FXP_EINVAL, "workspace must be 256-byte aligned");
    if (probs && probs_stride < 1) return fail(FXP_EINVAL, "probs_stride must be positive");
    Workspace w = carve(d, T, B, batch->max_blocks_per_seq, (char *)workspace);
    if (workspace_bytes < w.bytes) return fail(FXP_ENOSPC, "workspace too small: %zu < %zu", workspace_bytes, w.bytes);

    hipStream_t st = (hipStream_t)hip_stream;
    const int H = d.hidden, D = d.head_dim, Nq = d.n_q_heads * D, Nall = (d.n_q_heads + 2 * d.n_kv_heads) * D, F = d.ffn;
    const bool skinny = T <= kSkinnyMaxTokens;
    const bool decode = batch->max_q_len == 1 && T == B;
    // lengths live on the device: a ragged call with several sequences may mix prompt chunks and single-token rows
    // (unless the caller says that no sequence has fewer than two new tokens)
    const bool mixed = !decode && !probs && B >= 2 && batch->max_q_len > 1 && (int64_t)T < (int64_t)B * batch->max_q_len &&
                       batch->min_q_len < 2;
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)D);
    hipError_t e;

    const bool opt = d.arch == FXP_ARCH_OPT;
    // act_out: the projection applies its activation itself (no split-K): SwiGLU over gate|up tiles, or
    // relu(sum + act_bias) for an OPT-style feed-forward
    auto project_skinny = [&](const char *wbase, const uint16_t *X, int N, int K, int ldx, int *S_out, uint16_t *act_out = nullptr,
                              const uint16_t *act_bias = nullptr) -> hipError_t {
        if (T > kSkinnyWideTokens) {
            // 65..128 token rows: one 128-row tile of the tiled kernel covers the batch; split-K for parallelism
            fxp::TiledArgs t;
            t.W = (const uint16_t *)wbase; t.X = X; t.R = nullptr; t.C = nullptr; t.P = w.P; t.bias = nullptr; t.blk_m = 0; t.rope = fxp::RopeArgs{};
            t.M = T; t.K = K; t.KS = k_steps(K); t.NT = N / 16; t.ldx = ldx; t.ldc = 0; t.epilogue = fxp::kEpiPartial;
            t.S = skinny_cfg(N, K, T).S;
            *S_out = t.S;
            KernelTimer kt(kKcSkinny, st);
            return fxp::launch_gemm_tiled(t, st);
        }
        fxp::SkinnyArgs a;
        a.W = (const uint16_t *)wbase; a.X = X; a.P = w.P; a.A = nullptr; a.bias = nullptr; a.act = 0;
        a.M = T; a.N = N; a.K = K; a.KS = k_steps(K); a.NT = N / 16; a.ldx = ldx; a.S = skinny_cfg(N, K, T).S; a.R = skinny_cfg(N, K, T).R;
        // register ring of the weight stream (NB buffers of U k-steps), measured: four buffers of two k-steps
        // beat two of four everywhere up to 32 rows (7B shape: 96 -> 90 us per layer), in the unsplit form
        // with its long k range (13B shape, 64 rows: 62 -> 53 us), and at 33..64 rows once there is one workgroup
        // per CU (a shape whose registers do not allow four buffers falls back to two in the launcher)
        static const int forced_u = env_int("FXP_SKINNY_U", 0), forced_nb = env_int("FXP_SKINNY_NB", 0);
        a.U = forced_u ? forced_u : 2;
        a.NB = forced_nb ? forced_nb : 4;
        if (act_out) {       // activation in the epilogue: no split; for SwiGLU the gate and the up tile sit in one wavefront
            a.A = act_out; a.S = 1; a.R = 2;
            if (act_bias) { a.act = 1; a.bias = act_bias; }
        }
        *S_out = a.S;
        KernelTimer kt(kKcSkinny, st);
        return fxp::launch_gemm_skinny(a, st);
    };
    auto project_tiled = [&](const char *wbase, const uint16_t *X, int N, int K, int ldx, uint16_t *C, int ldc,
                             const uint16_t *R, int epi, const uint16_t *bias = nullptr, int kernel_class = kKcTiled) -> hipError_t {
        fxp::TiledArgs a;
        a.W = (const uint16_t *)wbase; a.X = X; a.R = R; a.C = C; a.P = nullptr; a.S = 1; a.bias = bias; a.blk_m = 0; a.rope = fxp::RopeArgs{};
        a.M = T; a.K = K; a.KS = k_steps(K); a.NT = N / 16; a.ldx = ldx; a.ldc = ldc; a.epilogue = epi;
        KernelTimer kt(kernel_class, st);
        return fxp::launch_gemm_tiled(a, st);
    };

    {   // token -> (sequence, position) and the rotation table: the same for every layer
        fxp::RopeTableArgs rt;
        rt.cu_seqlens_q = batch->cu_seqlens_q; rt.ctx_lens = batch->ctx_lens; rt.tok_seq = w.tok_seq; rt.tok_pos = w.tok_pos; rt.blk_prefix = w.blk_prefix;
        rt.tok_row = w.tok_row; rt.block_table = batch->block_table; rt.max_blocks_per_seq = batch->max_blocks_per_seq; rt.n_kv_heads = d.n_kv_heads;
        rt.cs = w.rope_cs; rt.sn = w.rope_sn; rt.T = T; rt.num_seqs = B; rt.head_dim = D; rt.rope_base = d.rope_base;
        rt.identity = opt ? 1 : 0;
        rt.one_token_each = decode ? 1 : 0;
        // the attention norm of the stage's first layer goes with it
        rt.norm_x = (const uint16_t *)hidden_in; rt.norm_g = (const uint16_t *)(stage->arena + stage->rec.g_attn);
        rt.norm_b = opt ? (const uint16_t *)(stage->arena + stage->rec.b_attn) : nullptr;
        rt.norm_out = w.n; rt.norm_H = H; rt.norm_eps = d.rms_eps;
        KernelTimer kt(kKcRopeTable, st);
        if ((e = fxp::launch_rope_table(rt, st))) return hip_fail(e, "rope table");
    }
    const uint16_t *x_cur = (const uint16_t *)hidden_in;
    bool n_ready = true;        // w.n holds the attention norm of the layer's input (the first layer's came with the rope table)
    for (int ll = 0; ll < stage->n_layers; ++ll) {
        const char *rec = stage->arena + stage->rec.bytes * (size_t)ll;
        const uint16_t *g_attn = (const uint16_t *)(rec + stage->rec.g_attn), *g_ffn = (const uint16_t *)(rec + stage->rec.g_ffn);
        auto vec = [&](size_t off) { return opt ? (const uint16_t *)(rec + off) : nullptr; };     // OPT-style biases, null otherwise
        const uint16_t *b_attn = vec(stage->rec.b_attn), *b_ffn = vec(stage->rec.b_ffn), *b_qkv = vec(stage->rec.b_qkv);
        const uint16_t *b_o = vec(stage->rec.b_o), *b_up = vec(stage->rec.b_up), *b_down = vec(stage->rec.b_down);
        const bool last = ll + 1 == stage->n_layers;
        uint16_t *x_next = last ? (uint16_t *)hidden_out : w.x[ll & 1];
        float *dbg = probs ? probs + (int64_t)ll * T * d.n_q_heads * probs_stride : nullptr;
        int S = 1;

        // Each projection either fills the chip by itself and finishes in its own epilogue (bf16 store, residual,
        // activation), or is split along k and leaves float partial sums that the row kernel behind it reduces
        // (together with rotary embedding / residual / norm / activation): always up to 128 rows, and above that
        // for matrices with too few tiles (a 4096-wide output has 16 x rows/128 of them).
        const int Nup = opt ? F : 2 * F;
        const bool part_qkv = skinny || skinny_cfg(Nall, H, T).S > 1;
        const bool part_o = skinny || skinny_cfg(H, Nq, T).S > 1;
        const bool part_down = skinny || skinny_cfg(H, F, T).S > 1;

        // attention norm (the first layer's came with the rope table; later ones come from the previous layer's
        // residual kernel when its down projection was split)
        if (!n_ready) {
            KernelTimer kt(kKcRmsnorm, st);
            if ((e = fxp::launch_rmsnorm(x_cur, g_attn, b_attn, w.n, T, H, d.rms_eps, st))) return hip_fail(e, "rmsnorm");
        }

        // q|k|v projection, rotary embedding, cache append
        fxp::RopeArgs ra;
        ra.P = nullptr; ra.qkv = nullptr; ra.S = 1; ra.bias = nullptr;
        if (part_qkv) {
            if ((e = project_skinny(rec + stage->rec.wqkv, w.n, Nall, H, H, &S))) return hip_fail(e, "qkv projection");
            ra.P = w.P; ra.S = S; ra.bias = b_qkv;
        }
        ra.q_out = w.q; ra.pool = (uint16_t *)pool->base;
        ra.tok_seq = w.tok_seq; ra.tok_pos = w.tok_pos; ra.tok_row = w.tok_row; ra.cs = w.rope_cs; ra.sn = w.rope_sn; ra.block_table = batch->block_table;
        ra.num_blocks = pool->num_blocks; ra.T = T; ra.max_blocks_per_seq = batch->max_blocks_per_seq;
        ra.layer_local = ll; ra.n_q_heads = d.n_q_heads; ra.n_kv_heads = d.n_kv_heads; ra.head_dim = D;
        bool qkv_done = false;
        if (!part_qkv) {
            // unsplit: on the wide tile the projection rotates q and k and appends k, v to the cache in its own epilogue;
            // otherwise it stores q|k|v as bf16 for the row kernel
            fxp::TiledArgs ta;
            ta.W = (const uint16_t *)(rec + stage->rec.wqkv); ta.X = w.n; ta.R = nullptr; ta.C = w.qkv; ta.P = nullptr; ta.S = 1; ta.bias = b_qkv;
            ta.blk_m = 0; ta.M = T; ta.K = H; ta.KS = k_steps(H); ta.NT = Nall / 16; ta.ldx = H; ta.ldc = Nall; ta.epilogue = fxp::kEpiRope;
            ta.rope = ra;
            if (fxp::gemm_wide_applies(ta)) {
                KernelTimer kt(kKcTiled, st);
                if ((e = fxp::launch_gemm_tiled(ta, st))) return hip_fail(e, "qkv projection + rope + kv append");
                qkv_done = true;
            } else {
                if ((e = project_tiled(rec + stage->rec.wqkv, w.n, Nall, H, H, w.qkv, Nall, nullptr, fxp::kEpiStore, b_qkv))) return hip_fail(e, "qkv projection");
                ra.qkv = w.qkv;
            }
        }
        if (!qkv_done) {
            KernelTimer kt(kKcRope, st);
            if ((e = fxp::launch_qkv_rope_kvwrite(ra, st))) return hip_fail(e, "rope + kv append");
        }

        // attention: sequences with one new token by the decode kernels, longer chunks by the prefill kernel (a call that
        // may hold both -- ragged, more than one sequence -- launches both; each leaves the other's sequences alone)
        if (decode || mixed) {
            fxp::DecodeAttnArgs aa;
            aa.q = w.q; aa.pool = (const uint16_t *)pool->base; aa.ctx_lens = batch->ctx_lens; aa.block_table = batch->block_table;
            aa.cu_seqlens_q = batch->cu_seqlens_q; aa.blk_prefix = w.blk_prefix;
            aa.part_acc = w.part_acc; aa.part_ml = w.part_ml; aa.out = w.o; aa.dbg_scores = dbg; aa.dbg_stride = probs_stride;
            aa.num_blocks = pool->num_blocks; aa.num_seqs = B; aa.max_blocks_per_seq = batch->max_blocks_per_seq;
            aa.n_workers = w.n_workers; aa.layer_local = ll; aa.n_q_heads = d.n_q_heads; aa.n_kv_heads = d.n_kv_heads;
            aa.head_dim = D; aa.scale_log2e = scale_log2e; aa.head_group = fxp::decode_head_group(d.n_kv_heads);
            {
                KernelTimer kt(kKcAttnDecode, st);
                if ((e = fxp::launch_attn_decode(aa, st))) return hip_fail(e, "decode attention");
            }
            {
                KernelTimer kt(kKcAttnCombine, st);
                if ((e = fxp::launch_attn_decode_combine(aa, st))) return hip_fail(e, "decode attention combine");
            }
        }
        if (!decode) {
            fxp::PrefillAttnArgs pa;
            pa.skip_single = mixed ? 1 : 0;
            pa.q = w.q; pa.pool = (const uint16_t *)pool->base; pa.cu_seqlens_q = batch->cu_seqlens_q; pa.ctx_lens = batch->ctx_lens;
            pa.block_table = batch->block_table; pa.out = w.o; pa.dbg_scores = dbg; pa.dbg_ml = w.dbg_ml; pa.dbg_stride = probs_stride;
            pa.num_blocks = pool->num_blocks; pa.num_seqs = B; pa.num_tokens = T; pa.max_q_len = batch->max_q_len;
            pa.max_blocks_per_seq = batch->max_blocks_per_seq; pa.layer_local = ll; pa.n_q_heads = d.n_q_heads;
            pa.n_kv_heads = d.n_kv_heads; pa.head_dim = D; pa.scale_log2e = scale_log2e;
            pa.tok_seq = w.tok_seq; pa.part_acc = w.pf_acc; pa.part_ml = w.pf_ml;
            pa.q_tile = fxp::prefill_q_tile(d.n_q_heads, T, B, batch->max_q_len, batch->max_blocks_per_seq);
            pa.kv_split = fxp::prefill_kv_split(d.n_q_heads, T, B, batch->max_blocks_per_seq, pa.q_tile);
            KernelTimer kt(kKcAttnPrefill, st);
            if ((e = fxp::launch_attn_prefill(pa, st))) return hip_fail(e, "prefill attention");
        }

        // output projection + residual, then the feed-forward norm
        fxp::ResidNormArgs rn;
        rn.T = T; rn.H = H; rn.eps = d.rms_eps; rn.P = w.P;
        if (part_o) {
            if ((e = project_skinny(rec + stage->rec.wo, w.o, H, Nq, Nq, &S))) return hip_fail(e, "output projection");
            rn.x = x_cur; rn.h = w.h; rn.g = g_ffn; rn.n = w.n; rn.S = S; rn.bias = b_o; rn.nb = b_ffn;
            KernelTimer kt(kKcResidNorm, st);
            if ((e = fxp::launch_resid_norm(rn, st))) return hip_fail(e, "residual + norm");
        } else {
            if ((e = project_tiled(rec + stage->rec.wo, w.o, H, Nq, Nq, w.h, H, x_cur, fxp::kEpiResidual, b_o))) return hip_fail(e, "output projection");
            KernelTimer kt(kKcRmsnorm, st);
            if ((e = fxp::launch_rmsnorm(w.h, g_ffn, b_ffn, w.n, T, H, d.rms_eps, st))) return hip_fail(e, "rmsnorm");
        }

        // gate|up projection + SwiGLU (an OPT-style layer has one matrix here and relu(sum + bias) as activation).
        // Up to 64 rows the weight-streaming kernel applies the activation itself when the matrix fills the chip
        // unsplit; above, the tiled kernel does when it is unsplit; split partial sums go through the activation kernel.
        {
            const bool tiled_unsplit = T > kSkinnyWideTokens && skinny_cfg(Nup, H, T).S == 1;
            const bool fused_act = tiled_unsplit || (T <= kSkinnyWideTokens && skinny_fused_swiglu(Nup));
            if (tiled_unsplit) {
                if ((e = project_tiled(rec + stage->rec.wgu, w.n, Nup, H, H, w.a, F, nullptr, opt ? fxp::kEpiRelu : fxp::kEpiSwiglu, b_up,
                                       skinny ? kKcSkinny : kKcTiled)))
                    return hip_fail(e, "gate/up projection");
            } else if ((e = project_skinny(rec + stage->rec.wgu, w.n, Nup, H, H, &S, fused_act ? w.a : nullptr, b_up))) {
                return hip_fail(e, "gate/up projection");
            }
            if (!fused_act) {
                fxp::SwigluArgs sg;
                sg.P = w.P; sg.out = w.a; sg.T = T; sg.F = F; sg.S = S; sg.ld_out = F; sg.bias = b_up; sg.act = opt ? 1 : 0;
                KernelTimer kt(kKcSwiglu, st);
                if ((e = fxp::launch_swiglu(sg, st))) return hip_fail(e, "swiglu");
            }
        }

        // down projection + residual; split: fused with the next layer's attention norm
        if (part_down) {
            if ((e = project_skinny(rec + stage->rec.wd, w.a, H, F, F, &S))) return hip_fail(e, "down projection");
            rn.x = w.h; rn.h = x_next; rn.S = S; rn.bias = b_down; rn.n = w.n;
            rn.g = last ? nullptr : (const uint16_t *)(rec + stage->rec.bytes + stage->rec.g_attn);
            rn.nb = (last || !opt) ? nullptr : (const uint16_t *)(rec + stage->rec.bytes + stage->rec.b_attn);
            KernelTimer kt(kKcResidNorm, st);
            if ((e = fxp::launch_resid_norm(rn, st))) return hip_fail(e, "residual + norm");
            n_ready = true;
        } else {
            if ((e = project_tiled(rec + stage->rec.wd, w.a, H, F, F, x_next, H, w.h, fxp::kEpiResidual, b_down))) return hip_fail(e, "down projection");
            n_ready = false;
        }
        x_cur = x_next;
    }
    return FXP_OK;
}

int fxp_stage_forward(fxp_stage *stage, const fxp_kv_pool *pool, const fxp_batch *batch, const void *hidden_in,
                      void *hidden_out, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return forward_impl(stage, pool, batch, hidden_in, hidden_out, workspace, workspace_bytes, nullptr, 0, hip_stream);
}

// ---- the forward step for callers that cannot allocate: the workspace is a file-scope device array.
// The array's name is only a host-side stand-in; its address on the current device comes from
// hipGetSymbolAddress, once per device, and that pointer is what the kernels get.
static __device__ __align__(256) unsigned char scratch[FXP_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mutex;

int static_scratch(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(FXP_EINVAL, "device index %d out of range", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if ((e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        if (!p || (uintptr_t)p % 256) return fail(FXP_EHIP, "static scratch has no usable device address");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return FXP_OK;
}
}  // namespace

int fxp_stage_forward_static(fxp_stage *stage, const fxp_kv_pool *pool, const fxp_batch *batch, const void *hidden_in,
                             void *hidden_out, void *hip_stream)
{
    if (!stage || !pool || !batch) return fail(FXP_EINVAL, "null argument to fxp_stage_forward_static");
    if (batch->num_tokens < 0 || batch->num_seqs < 0) return fail(FXP_EINVAL, "negative batch size");
    if (batch->num_seqs > FXP_MAX_SEQS) return fail(FXP_EINVAL, "num_seqs %d above the limit of %d", batch->num_seqs, FXP_MAX_SEQS);
    const size_t need = carve(stage->d, batch->num_tokens, batch->num_seqs, batch->max_blocks_per_seq, nullptr).bytes;
    if (need > (size_t)FXP_STATIC_SCRATCH_BYTES)
        return fail(FXP_ENOSPC, "a step of %d tokens and %d sequences needs %zu bytes of scratch; the static scratch holds %zu "
                                "(use fxp_stage_forward with a workspace of the caller's)",
                    batch->num_tokens, batch->num_seqs, need, (size_t)FXP_STATIC_SCRATCH_BYTES);
    void *ws = nullptr;
    if (int rc = static_scratch(&ws)) return rc;
    return forward_impl(stage, pool, batch, hidden_in, hidden_out, ws, (size_t)FXP_STATIC_SCRATCH_BYTES, nullptr, 0, hip_stream);
}

int fxp_stage_forward_debug(fxp_stage *stage, const fxp_kv_pool *pool, const fxp_batch *batch, const void *hidden_in,
                            void *hidden_out, void *workspace, size_t workspace_bytes, float *probs,
                            int64_t probs_stride, void *hip_stream)
{
    if (!probs) return fail(FXP_EINVAL, "probs is null");
    return forward_impl(stage, pool, batch, hidden_in, hidden_out, workspace, workspace_bytes, probs, probs_stride, hip_stream);
}

// ------------------------------------------------------------------ KV repartition

static int check_view(const fxp_kv_view *v, const char *what, int idx)
{
    if (!v->pool || !v->pool->base || !v->block_table) return fail(FXP_EINVAL, "%s view %d has a null pointer", what, idx);
    if (v->pool->num_blocks <= 0 || v->max_blocks_per_seq <= 0) return fail(FXP_EINVAL, "%s view %d is empty", what, idx);
    if (v->pool->layer_begin < 0 || v->pool->layer_end <= v->pool->layer_begin) return fail(FXP_EINVAL, "%s view %d has a bad layer range", what, idx);
    return FXP_OK;
}

static int check_tiling(const fxp_kv_view *v, int n, const char *what)
{
    for (int i = 0; i < n; ++i) if (int rc = check_view(&v[i], what, i)) return rc;
    for (int i = 1; i < n; ++i)
        if (v[i].pool->layer_begin != v[i - 1].pool->layer_end)
            return fail(FXP_EINVAL, "%s views do not tile a layer range (view %d starts at %d, previous ends at %d)", what, i,
                        v[i].pool->layer_begin, v[i - 1].pool->layer_end);
    return FXP_OK;
}

static fxp::KvMoveSide pool_side(const fxp_kv_view &v)
{
    fxp::KvMoveSide s;
    s.base = (char *)v.pool->base; s.table = v.block_table; s.num_blocks = v.pool->num_blocks; s.limit_bytes = 0;
    s.layer_base = v.pool->layer_begin; s.n_layers = v.pool->layer_end - v.pool->layer_begin; s.max_blocks_per_seq = v.max_blocks_per_seq;
    s.token_dense = 0;
    return s;
}

static fxp::KvMoveSide packed_side(const void *buf, size_t bytes, int lb, int le, bool token_dense = false)
{
    fxp::KvMoveSide s;
    s.base = (char *)buf; s.table = nullptr; s.num_blocks = 0; s.limit_bytes = (int64_t)bytes;
    s.layer_base = lb; s.n_layers = le - lb; s.max_blocks_per_seq = 0;
    s.token_dense = token_dense ? 1 : 0;
    return s;
}

static int move_grid(const fxp::KvMoveArgs &a, int max_blocks_per_seq)
{
    const int64_t chunks = (a.unit_bytes + fxp::kv_move_chunk_bytes() - 1) / fxp::kv_move_chunk_bytes();
    int64_t items = 0;
    for (int j = 0; j < a.n_jobs; ++j)
        items += (int64_t)a.num_seqs * max_blocks_per_seq * (a.jobs[j].layer_end - a.jobs[j].layer_begin) * chunks;
    // persistent grid: as many workgroups as are resident (the token-dense variant needs more registers)
    const bool dense = a.n_jobs > 0 && (a.jobs[0].src.token_dense || a.jobs[0].dst.token_dense);
    int64_t grid = (int64_t)device_cus() * (dense ? 4 : env_int("FXP_MOVE_WGS_PER_CU", 8));
    if (grid > items) grid = items;
    return (int)(grid < 1 ? 1 : grid);
}

static int launch_moves(fxp::KvMoveArgs &a, int max_blocks_per_seq, hipStream_t st)
{
    if (a.n_jobs == 0) return FXP_OK;
    KernelTimer kt(kKcKvMove, st);
    hipError_t e = fxp::launch_kv_move(a, move_grid(a, max_blocks_per_seq), st);
    if (e != hipSuccess) return hip_fail(e, "kv move");
    return FXP_OK;
}

static int repartition_impl(const fxp_stage_desc *desc, const fxp_kv_view *src, int32_t n_src, const fxp_kv_view *dst,
                            int32_t n_dst, const int32_t *from_lens, const int32_t *ctx_lens, int32_t num_seqs, void *hip_stream)
{
    if (int rc = check_kv_geom(desc)) return rc;
    if (!src || !dst || n_src <= 0 || n_dst <= 0) return fail(FXP_EINVAL, "empty view list");
    if (num_seqs < 0 || num_seqs > FXP_MAX_SEQS) return fail(FXP_EINVAL, "num_seqs %d out of range [0,%d]", num_seqs, FXP_MAX_SEQS);
    if (int rc = check_tiling(src, n_src, "source")) return rc;
    if (int rc = check_tiling(dst, n_dst, "destination")) return rc;
    if (src[0].pool->layer_begin != dst[0].pool->layer_begin || src[n_src - 1].pool->layer_end != dst[n_dst - 1].pool->layer_end)
        return fail(FXP_EINVAL, "source layers [%d,%d) and destination layers [%d,%d) differ", src[0].pool->layer_begin,
                    src[n_src - 1].pool->layer_end, dst[0].pool->layer_begin, dst[n_dst - 1].pool->layer_end);
    const int64_t unit = 2ll * desc->n_kv_heads * 16 * desc->head_dim * 2;
    for (int s = 0; s < n_src; ++s)
        for (int t = 0; t < n_dst; ++t) {
            const char *sb = (const char *)src[s].pool->base, *db = (const char *)dst[t].pool->base;
            const int64_t sbytes = unit * src[s].pool->num_blocks * (src[s].pool->layer_end - src[s].pool->layer_begin);
            const int64_t dbytes = unit * dst[t].pool->num_blocks * (dst[t].pool->layer_end - dst[t].pool->layer_begin);
            if (sb < db + dbytes && db < sb + sbytes) return fail(FXP_EINVAL, "source pool %d overlaps destination pool %d", s, t);
        }
    if (num_seqs == 0) return FXP_OK;
    if (!ctx_lens) return fail(FXP_EINVAL, "ctx_lens is null");

    fxp::KvMoveArgs a;
    a.from_lens = from_lens; a.to_lens = ctx_lens; a.unit_bytes = unit; a.num_seqs = num_seqs; a.head_dim = desc->head_dim; a.n_jobs = 0;
    int max_blocks = 0;
    for (int t = 0; t < n_dst; ++t)
        for (int s = 0; s < n_src; ++s) {
            const int lb = src[s].pool->layer_begin > dst[t].pool->layer_begin ? src[s].pool->layer_begin : dst[t].pool->layer_begin;
            const int le = src[s].pool->layer_end < dst[t].pool->layer_end ? src[s].pool->layer_end : dst[t].pool->layer_end;
            if (lb >= le) continue;
            if (a.n_jobs == fxp::kMaxMoveJobs) {
                if (int rc = launch_moves(a, max_blocks, (hipStream_t)hip_stream)) return rc;
                a.n_jobs = 0; max_blocks = 0;
            }
            fxp::KvMoveJob &j = a.jobs[a.n_jobs++];
            j.src = pool_side(src[s]); j.dst = pool_side(dst[t]); j.layer_begin = lb; j.layer_end = le;
            const int mb = src[s].max_blocks_per_seq < dst[t].max_blocks_per_seq ? src[s].max_blocks_per_seq : dst[t].max_blocks_per_seq;
            if (mb > max_blocks) max_blocks = mb;
        }
    return launch_moves(a, max_blocks, (hipStream_t)hip_stream);
}

int fxp_kv_repartition(const fxp_stage_desc *desc, const fxp_kv_view *src, int32_t n_src, const fxp_kv_view *dst,
                       int32_t n_dst, const int32_t *ctx_lens, int32_t num_seqs, void *hip_stream)
{
    return repartition_impl(desc, src, n_src, dst, n_dst, nullptr, ctx_lens, num_seqs, hip_stream);
}

int fxp_kv_repartition_range(const fxp_stage_desc *desc, const fxp_kv_view *src, int32_t n_src, const fxp_kv_view *dst,
                             int32_t n_dst, const int32_t *from_lens, const int32_t *to_lens, int32_t num_seqs, void *hip_stream)
{
    if (num_seqs > 0 && !from_lens) return fail(FXP_EINVAL, "from_lens is null");
    return repartition_impl(desc, src, n_src, dst, n_dst, from_lens, to_lens, num_seqs, hip_stream);
}

size_t fxp_kv_packed_bytes(const fxp_stage_desc *desc, int32_t layer_begin, int32_t layer_end,
                           const int32_t *ctx_lens_host, int32_t num_seqs)
{
    if (check_kv_geom(desc) != FXP_OK) return 0;
    if (layer_begin < 0 || layer_end <= layer_begin || num_seqs < 0 || (num_seqs > 0 && !ctx_lens_host)) {
        fail(FXP_EINVAL, "bad argument to fxp_kv_packed_bytes");
        return 0;
    }
    size_t blocks = 0;
    for (int i = 0; i < num_seqs; ++i) blocks += (size_t)((ctx_lens_host[i] + 15) / 16);
    return blocks * (size_t)(layer_end - layer_begin) * 2 * desc->n_kv_heads * 16 * desc->head_dim * 2;
}

static int pack_or_unpack(const fxp_stage_desc *desc, const fxp_kv_view *view, int lb, int le, const int32_t *from_lens,
                          const int32_t *ctx_lens, int num_seqs, void *packed, size_t packed_bytes, bool to_packed,
                          bool token_dense, void *hip_stream)
{
    if (int rc = check_kv_geom(desc)) return rc;
    if (!view) return fail(FXP_EINVAL, "view is null");
    if (int rc = check_view(view, to_packed ? "source" : "destination", 0)) return rc;
    if (lb < view->pool->layer_begin || le > view->pool->layer_end || lb >= le)
        return fail(FXP_EINVAL, "layers [%d,%d) are not inside the pool's [%d,%d)", lb, le, view->pool->layer_begin, view->pool->layer_end);
    if (num_seqs < 0 || num_seqs > FXP_MAX_SEQS) return fail(FXP_EINVAL, "num_seqs %d out of range [0,%d]", num_seqs, FXP_MAX_SEQS);
    if (num_seqs == 0) return FXP_OK;
    if (!ctx_lens || !packed || (token_dense && !from_lens)) return fail(FXP_EINVAL, "null buffer");
    const int64_t unit = 2ll * desc->n_kv_heads * 16 * desc->head_dim * 2;
    if (token_dense) {
        if (packed_bytes < 16) return fail(FXP_ENOSPC, "packed buffer smaller than one vector");
    } else if (packed_bytes < (size_t)unit * (size_t)(le - lb)) {
        return fail(FXP_ENOSPC, "packed buffer smaller than one block per layer");
    }
    fxp::KvMoveArgs a;
    a.from_lens = from_lens; a.to_lens = ctx_lens; a.unit_bytes = unit; a.num_seqs = num_seqs; a.head_dim = desc->head_dim; a.n_jobs = 1;
    fxp::KvMoveJob &j = a.jobs[0];
    j.layer_begin = lb; j.layer_end = le;
    if (to_packed) { j.src = pool_side(*view); j.dst = packed_side(packed, packed_bytes, lb, le, token_dense); }
    else           { j.src = packed_side(packed, packed_bytes, lb, le, token_dense); j.dst = pool_side(*view); }
    return launch_moves(a, view->max_blocks_per_seq, (hipStream_t)hip_stream);
}

int fxp_kv_pack(const fxp_stage_desc *desc, const fxp_kv_view *src, int32_t layer_begin, int32_t layer_end,
                const int32_t *ctx_lens, int32_t num_seqs, void *packed, size_t packed_bytes, void *hip_stream)
{
    return pack_or_unpack(desc, src, layer_begin, layer_end, nullptr, ctx_lens, num_seqs, packed, packed_bytes, true, false, hip_stream);
}

int fxp_kv_unpack(const fxp_stage_desc *desc, const void *packed, size_t packed_bytes, const fxp_kv_view *dst,
                  int32_t layer_begin, int32_t layer_end, const int32_t *ctx_lens, int32_t num_seqs, void *hip_stream)
{
    return pack_or_unpack(desc, dst, layer_begin, layer_end, nullptr, ctx_lens, num_seqs, const_cast<void *>(packed), packed_bytes, false, false, hip_stream);
}

size_t fxp_kv_packed_tokens_bytes(const fxp_stage_desc *desc, int32_t layer_begin, int32_t layer_end,
                                  const int32_t *from_lens_host, const int32_t *to_lens_host, int32_t num_seqs)
{
    if (check_kv_geom(desc) != FXP_OK) return 0;
    if (layer_begin < 0 || layer_end <= layer_begin || num_seqs < 0 || (num_seqs > 0 && (!from_lens_host || !to_lens_host))) {
        fail(FXP_EINVAL, "bad argument to fxp_kv_packed_tokens_bytes");
        return 0;
    }
    size_t tokens = 0;
    for (int i = 0; i < num_seqs; ++i)
        if (from_lens_host[i] >= 0 && to_lens_host[i] > from_lens_host[i]) tokens += (size_t)(to_lens_host[i] - from_lens_host[i]);
    return tokens * (size_t)(layer_end - layer_begin) * 2 * desc->n_kv_heads * desc->head_dim * 2;
}

int fxp_kv_pack_tokens(const fxp_stage_desc *desc, const fxp_kv_view *src, int32_t layer_begin, int32_t layer_end,
                       const int32_t *from_lens, const int32_t *to_lens, int32_t num_seqs, void *packed, size_t packed_bytes,
                       void *hip_stream)
{
    return pack_or_unpack(desc, src, layer_begin, layer_end, from_lens, to_lens, num_seqs, packed, packed_bytes, true, true, hip_stream);
}

int fxp_kv_unpack_tokens(const fxp_stage_desc *desc, const void *packed, size_t packed_bytes, const fxp_kv_view *dst,
                         int32_t layer_begin, int32_t layer_end, const int32_t *from_lens, const int32_t *to_lens,
                         int32_t num_seqs, void *hip_stream)
{
    return pack_or_unpack(desc, dst, layer_begin, layer_end, from_lens, to_lens, num_seqs, const_cast<void *>(packed), packed_bytes,
                          false, true, hip_stream);
}

}  // extern "C"
