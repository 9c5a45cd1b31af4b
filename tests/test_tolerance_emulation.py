"""Where the stated tolerances sit relative to bf16 rounding alone.

The tolerances (stage outputs 2e-2, probabilities 1e-3) are given by the task,
not by the paper.  This test replays one decode step of the tiny configuration
with the oracle's own double-precision operations, but rounds to bf16 at the
points where the GPU path stores bf16 (norm output, rotated q, appended K/V,
attention output, hidden after each residual, SwiGLU output).  The resulting
error against the unrounded oracle is what ANY bf16-storage pipeline must show;
it has to sit well inside the tolerance for the tolerance to be meaningful."""
import numpy as np
import pytest

import oracle
from oracle import Shape
from paper_2510_11938_amd import synth

import wide_tolerance as wt


def bf16(x):
    return synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))).astype(np.float64)


def emulated_decode(sh, layers, pool, ctx, table, x):
    """One decode token per sequence; float64 arithmetic, bf16 storage points."""
    B = len(ctx)
    D, Hq, Hkv = sh.head_dim, sh.n_q_heads, sh.n_kv_heads
    probs_all = []
    for ll, L in enumerate(layers):
        n = bf16(oracle.rmsnorm(x, L["g_attn"], sh.rms_eps))
        q = oracle.linear(n, L["wq"]).reshape(B, Hq, D)
        k = oracle.linear(n, L["wk"]).reshape(B, Hkv, D)
        v = oracle.linear(n, L["wv"]).reshape(B, Hkv, D)
        o = np.zeros((B, Hq * D))
        layer_probs = []
        for i in range(B):
            p = int(ctx[i])
            qi = bf16(np.stack([oracle.rope(q[i, h], p, sh.rope_base) for h in range(Hq)]))
            ki = bf16(np.stack([oracle.rope(k[i, h], p, sh.rope_base) for h in range(Hkv)]))
            pool[ll, table[i, p // 16], 0, :, p % 16, :] = ki
            pool[ll, table[i, p // 16], 1, :, p % 16, :] = bf16(v[i])
            oi, pr = oracle.attend_token(sh, pool, ll, table[i], p, qi, want_probs=True)
            o[i] = bf16(oi).reshape(-1)
            layer_probs.append(pr)
        h = bf16(x + oracle.linear(o, L["wo"]))
        m = bf16(oracle.rmsnorm(h, L["g_ffn"], sh.rms_eps))
        g, u = oracle.linear(m, L["w_gate"]), oracle.linear(m, L["w_up"])
        a = bf16(g / (1.0 + np.exp(-g)) * u)
        x = bf16(h + oracle.linear(a, L["w_down"]))
        probs_all.append(layer_probs)
    return x, probs_all


def test_bf16_storage_alone_sits_well_inside_the_stated_tolerances():
    ms = synth.TINY
    sh = Shape(ms.hidden, ms.n_q_heads, ms.n_kv_heads, ms.head_dim, ms.ffn, 16, ms.rms_eps, ms.rope_base)
    Lr = 2
    layers = [{k: synth.bf16_bits_to_f32(v) for k, v in synth.layer_weights(ms, 11, l).items()} for l in range(Lr)]
    ctx = np.array([37, 128, 32, 100], dtype=np.int32)
    table, nblk = synth.block_table(ctx + 1, 16, 11)
    pool = oracle.new_pool(sh, Lr, nblk)
    for l in range(Lr):
        for i, c in enumerate(ctx):
            rows = synth.bf16_bits_to_f32(synth.cache_rows(ms, 11, i, l, int(c)))
            synth.fill_pool_rows(pool, l, table[i], rows, 16)
    x = synth.bf16_bits_to_f32(synth.hidden_states(len(ctx), ms.hidden, 11)).astype(np.float64)
    stride = int(ctx.max()) + 1
    want, want_probs = oracle.stage_forward(sh, layers, pool.copy(), np.arange(len(ctx) + 1), ctx, table, x, probs_stride=stride)
    got, got_probs = emulated_decode(sh, layers, pool.copy(), ctx, table, x)
    rms = np.sqrt((want ** 2).mean(axis=1, keepdims=True))
    err = float((np.abs(got - want) / np.maximum(np.abs(want), rms)).max())
    perr = max(float(np.abs(got_probs[l][i] - want_probs[l, i, :, : ctx[i] + 1]).max()) for l in range(Lr) for i in range(len(ctx)))
    print(f"bf16-storage emulation: output error {err:.2e} (tolerance 2e-2), probability error {perr:.2e} (tolerance 1e-3)")
    assert 1e-4 < err < 1.2e-2          # visible, and at most ~half of the tolerance
    assert perr < 5e-4


# ---- full width and depth ----------------------------------------------------------------------
# The same emulation at the widths and depths of the benchmark workloads (7B x 4 layers, 13B x 8, 70B x 4),
# four decode rows each.  It shows that the element-wise 2e-2 cannot hold at depth for ANY pipeline that
# stores bf16 where this one does, pins the figures the full-width GPU bar is derived from
# (wide_tolerance.EMULATED), and checks the relation the element-wise bar rests on.

@pytest.mark.slow
@pytest.mark.parametrize("name", list(wt.EMULATED_RUNS))
def test_bf16_storage_emulation_at_full_width_and_depth_gives_the_bar_of_the_gpu_tests(name):
    run = wt.EMULATED_RUNS[name]
    ms, depth = run["shape"], len(run["l2"])
    ctx = np.random.default_rng(5).integers(512, 800, size=4).astype(np.int32)
    res = wt.emulated_decode_errors(ms, depth, ctx, run["seed"])
    for k, r in enumerate(res):
        l2_rec, frac_rec = wt.EMULATED[("decode", ms.hidden, k + 1)]
        print(f"{name} after {k + 1} layers: row L2 {r['l2']:.3e} (recorded {l2_rec:.3e})  element-wise max {r['elem']:.3e}  "
              f"fraction > 2e-2 {r['frac']:.2e} (recorded {frac_rec:.2e})")
        # the recorded figures are these figures (2 % slack for a different libm or thread count)
        assert abs(r["l2"] - l2_rec) <= 0.02 * l2_rec
        assert abs(r["frac"] - frac_rec) <= 0.05 * frac_rec + 2e-4
        # the relation behind the element-wise bar: max over n elements below row L2 x sqrt(2 ln 2n)
        assert r["elem"] <= r["l2"] * wt.gaussian_max_factor(r["n"])
        # so the bar of the GPU tests leaves the emulation MARGIN_L2 of head room and no more
        l2_bar, elem_bar, frac_bar = wt.wide_bar(ms.hidden, k + 1, r["n"])
        assert r["l2"] <= l2_bar / 1.2 and r["elem"] <= elem_bar / 1.2 and r["frac"] <= frac_bar
    # storage rounding alone passes the element-wise 2e-2 at the full depth of every workload
    assert res[-1]["elem"] > 2e-2 and res[0]["elem"] < 2e-2


@pytest.mark.slow
@pytest.mark.parametrize("name", list(wt.EMULATED_PREFILL_RUNS))
def test_bf16_storage_emulation_of_a_prompt_gives_the_bar_of_the_prefill_tests(name):
    run = wt.EMULATED_PREFILL_RUNS[name]
    ms, depth = run["shape"], len(run["l2"])
    res = wt.emulated_prefill_errors(ms, depth, run["tokens"], run["seed"])
    for k, r in enumerate(res):
        l2_rec, frac_rec = wt.EMULATED[("prefill", ms.hidden, k + 1)]
        print(f"{name} prompt after {k + 1} layers: row L2 {r['l2']:.3e} (recorded {l2_rec:.3e}, worst row {int(r['l2_rows'].argmax())})  "
              f"element-wise max {r['elem']:.3e}  fraction > 2e-2 {r['frac']:.2e} (recorded {frac_rec:.2e})")
        assert abs(r["l2"] - l2_rec) <= 0.02 * l2_rec
        assert abs(r["frac"] - frac_rec) <= 0.05 * frac_rec + 2e-4
        assert r["elem"] <= r["l2"] * wt.gaussian_max_factor(r["n"])
        l2_bar, elem_bar, frac_bar = wt.wide_bar(ms.hidden, k + 1, r["n"], "prefill")
        assert r["l2"] <= l2_bar / 1.2 and r["elem"] <= elem_bar / 1.2 and r["frac"] <= frac_bar
        # the worst rows are early ones and the error falls off behind them, so 48 rows stand for a prompt of any length
        assert r["l2_rows"].argmax() < 40 and r["l2_rows"][40:].max() < r["l2"]
        # larger than a decode row's behind a long context at the same depth
        assert r["l2"] > wt.EMULATED[("decode", ms.hidden, k + 1)][0]
