"""Full-size parity: the benchmark workloads at their real width, batch AND depth (7B x 4 layers
decode and prefill, 13B x 8 layers, 70B grouped-query x 4 layers), in the launch configuration
bench.py times.  The GPU runs the whole batch; the oracle recomputes sampled sequences from the same
bits (batch rows are independent, and causal attention makes a prompt independent of its neighbours).
The cache of the big decode workloads is filled on the device (N(0,1) bf16 rows from torch's seeded
device generator) and only the sampled sequences' blocks are copied back for the oracle, so the
host never has to draw tens of gigabytes.  Outputs are judged by the bar derived from the
bf16-storage emulation (wide_tolerance.py)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_11938_amd import binding, synth

from gpu_util import dev_bf16, dev_i32, host_bits, host_f64, make_stage, make_weights, oracle_shape
from wide_tolerance import check_wide_output

pytestmark = pytest.mark.gpu


def device_filled_pool(ms, n_layers, nblk, seed):
    """[layers][blocks][2][Hkv][16][D] bf16 on the device, every slot N(0,1) (slots past a sequence's
    length are never read: attention stops at the length, repartition masks them)."""
    g = torch.Generator(device="cuda")
    g.manual_seed(1000 + seed)
    pool = torch.empty((n_layers, nblk, 2, ms.n_kv_heads, 16, ms.head_dim), dtype=torch.bfloat16, device="cuda")
    for l in range(n_layers):
        pool[l].normal_(generator=g)
    return pool.view(torch.int16)


def run_sampled_decode(wl_name, samples):
    wl = synth.WORKLOADS[wl_name]
    ms, L, B = wl.shape, wl.n_layers, wl.num_seqs
    ctx = synth.draw_lengths(wl.length_dist, B, wl.seed)
    table, nblk = synth.block_table(ctx + 1, 16, wl.seed)
    print(f"{wl_name}: {L} layers, batch {B}, {int(ctx.sum())} cached tokens; drawing weights", flush=True)
    w = make_weights(ms, wl.seed, L, want_f32=False)
    stage = make_stage(ms, w, 0, L)
    torch.cuda.synchronize()
    w.dev.clear()                                           # the stage keeps its own re-tiled copy
    cache = binding.KVCache(device_filled_pool(ms, L, nblk, wl.seed), 0, L, dev_i32(table))
    picks = sorted({int(np.argmin(ctx)), int(np.argmax(ctx)), *samples})
    nb = [(int(ctx[i]) + 16) // 16 for i in picks]
    table_dev = cache.block_table.long()
    sub_pool_bits = np.concatenate([host_bits(cache.pool[:, table_dev[i, :n]]) for i, n in zip(picks, nb)], axis=1)   # before the step appends
    hidden_bits = synth.hidden_states(B, ms.hidden, wl.seed)
    print(f"{wl_name}: GPU step", flush=True)
    y = stage.forward(cache, dev_i32(np.arange(B + 1)), dev_i32(ctx), dev_bf16(hidden_bits), 1)
    torch.cuda.synchronize()
    got = host_f64(y)
    assert np.isfinite(got).all()
    # the oracle on the sampled sequences alone, their blocks renumbered 0..n-1 one sequence after the other
    sub_table = np.full((len(picks), max(nb)), -1, dtype=np.int32)
    at = 0
    for r, n in enumerate(nb):
        sub_table[r, :n] = np.arange(at, at + n); at += n
    print(f"{wl_name}: oracle on sequences {picks} (contexts {[int(ctx[i]) for i in picks]})", flush=True)
    wf = [{k: synth.bf16_bits_to_f32(v) for k, v in lw.items()} for lw in w.bits]
    sub_pool = synth.bf16_bits_to_f32(sub_pool_bits)
    want = oracle.stage_forward(oracle_shape(ms), wf, sub_pool, np.arange(len(picks) + 1), ctx[picks], sub_table,
                                synth.bf16_bits_to_f32(hidden_bits[picks]).astype(np.float64))
    del wf
    for r, i in enumerate(picks):
        check_wide_output(got[i:i + 1], want[r:r + 1], ms.hidden, L, f"{wl_name} sequence {i} ctx {ctx[i]}:")
    # the K and V rows the step appended for the sampled sequences: bf16 roundings of the oracle's
    after = synth.bf16_bits_to_f32(host_bits(cache.pool[:, table_dev[picks[0], :nb[0]]])).astype(np.float64)
    p = int(ctx[picks[0]])
    g_rows = after[:, p // 16, :, :, p % 16, :].reshape(L * 2 * ms.n_kv_heads, ms.head_dim)
    o_rows = sub_pool[:, sub_table[0, p // 16], :, :, p % 16, :].astype(np.float64).reshape(g_rows.shape)
    scale = np.sqrt((o_rows ** 2).mean(axis=-1, keepdims=True))
    assert (np.abs(g_rows - o_rows) / np.maximum(np.abs(o_rows), scale)).max() <= 2 * check_bar(ms.hidden, L)
    return ms, ctx, cache, (picks, nb, sub_pool_bits, sub_table)


def check_bar(hidden, n_layers):
    from wide_tolerance import wide_bar
    return wide_bar(hidden, n_layers, hidden)[1]


def test_7b_shape_decode_batch_32_full_depth_sampled_against_oracle():
    # the benchmark's headline workload: hidden 4096, 32 x 128 heads, ffn 11008, 4 layers, batch 32, contexts U[512,4096]
    run_sampled_decode("C2", samples=[5])


def test_70b_gqa_shape_decode_batch_128_full_depth_sampled_against_oracle():
    # hidden 8192, 64 query / 8 kv heads x 128, ffn 28672, 4 layers, batch 128, contexts U[1024,8192]
    run_sampled_decode("C5", samples=[17])


def test_13b_shape_decode_batch_64_full_depth_then_resplit_sampled_against_oracle():
    # hidden 5120, 40 x 128 heads, ffn 13824, 8 layers, batch 64, lognormal contexts; then the inflight refactor of the
    # workload: the 8-layer stage's cache re-split 8 -> 4 + 4 into fresh permuted tables
    ms, ctx, cache, sampled = run_sampled_decode("C4", samples=[5])
    L = cache.layer_end
    lens = ctx + 1                                           # the step appended one token per sequence
    dst = []
    for s, (a, b) in enumerate([(0, L // 2), (L // 2, L)]):
        t, n = synth.block_table(lens, 16, 3, salt=7 + s, spare_blocks=2)
        dst.append(binding.KVCache(torch.full((b - a, n, 2, ms.n_kv_heads, 16, ms.head_dim), 0x2222, dtype=torch.int16, device="cuda"),
                                   a, b, dev_i32(t)))
    binding.kv_repartition(ms, [cache], dst, dev_i32(lens))
    torch.cuda.synchronize()
    nblk = (lens + 15) // 16
    src_pool = cache.pool.view(torch.int16)
    for dv in dst:
        owned = torch.zeros(dv.pool.shape[1], dtype=torch.bool, device="cuda")
        for i in range(len(lens)):
            sb = cache.block_table[i, : nblk[i]].long(); db = dv.block_table[i, : nblk[i]].long()
            owned[db] = True
            want = src_pool[dv.layer_begin:dv.layer_end][:, sb].clone()
            tail = int(lens[i] % 16)
            if tail:
                want[:, -1, :, :, tail:, :] = 0
            assert torch.equal(dv.pool[:, db], want), f"layers [{dv.layer_begin},{dv.layer_end}) sequence {i}"
        assert bool((dv.pool[:, ~owned] == 0x2222).all())
    # the sampled sequences against the oracle's repartition of their blocks as they were BEFORE the step (inputs only):
    # every token below the old length bit for bit; the appended token's row was checked above; slots behind it zero
    picks, nb, sub_pool_bits, sub_table = sampled
    o_dst = [np.full((dv.layer_end - dv.layer_begin, sub_pool_bits.shape[1], 2, ms.n_kv_heads, 16, ms.head_dim), 0x2222, dtype=np.uint16)
             for dv in dst]
    oracle.kv_repartition(oracle_shape(ms), [oracle.KVView(sub_pool_bits, 0, L, sub_table)],
                          [oracle.KVView(o, dv.layer_begin, dv.layer_end, sub_table) for o, dv in zip(o_dst, dst)], ctx[picks])
    for r, i in enumerate(picks):
        full, part = int(ctx[i]) // 16, int(ctx[i]) % 16
        for o, dv in zip(o_dst, dst):
            got = host_bits(dv.pool[:, dv.block_table[i, : nb[r]].long()])
            want = o[:, sub_table[r, : nb[r]]]
            assert np.array_equal(got[:, :full], want[:, :full]), f"sequence {i}: whole blocks against the oracle"
            assert np.array_equal(got[:, full, :, :, :part], want[:, full, :, :, :part]), f"sequence {i}: last block against the oracle"
            assert not got[:, full, :, :, part + 1:].any(), f"sequence {i}: slots behind the last token"


def test_7b_shape_prefill_chunk_of_514_tokens_sampled_against_oracle():
    # hidden 4096, 32 x 128 heads, ffn 11008; three prompts of 300 + 150 + 64 tokens in one call, 1 layer: between 128 and
    # 1024 rows the narrow projections (o, down) are split along k and finished by the row kernels, the wide ones are not
    ms = synth.WORKLOADS["C3"].shape
    seed, lens = 21, np.array([300, 150, 64], dtype=np.int32)
    T = int(lens.sum())
    table, nblk = synth.block_table(lens, 16, seed)
    w = make_weights(ms, seed, 1, want_f32=False)
    hidden_bits = synth.hidden_states(T, ms.hidden, seed)
    stage = make_stage(ms, w, 0, 1)
    pool = torch.zeros((1, nblk, 2, ms.n_kv_heads, 16, ms.head_dim), dtype=torch.int16, device="cuda")
    cache = binding.KVCache(pool, 0, 1, dev_i32(table))
    cu = synth.cu_seqlens(lens)
    y = stage.forward(cache, dev_i32(cu), dev_i32(np.zeros(3)), dev_bf16(hidden_bits), int(lens.max()))
    torch.cuda.synchronize()
    got = host_f64(y)
    assert np.isfinite(got).all()
    osh = oracle_shape(ms)
    wf = [{k: synth.bf16_bits_to_f32(v) for k, v in lw.items()} for lw in w.bits]
    for i in (2, 1):                                        # prompts are independent: the oracle recomputes two of them alone
        nb = (int(lens[i]) + 15) // 16
        sub_pool = np.zeros((1, nb, 2, ms.n_kv_heads, 16, ms.head_dim), dtype=np.float32)
        rows = slice(int(cu[i]), int(cu[i + 1]))
        want = oracle.stage_forward(osh, wf, sub_pool, [0, int(lens[i])], [0], np.arange(nb, dtype=np.int32)[None, :],
                                    synth.bf16_bits_to_f32(hidden_bits[rows]).astype(np.float64))
        check_wide_output(got[rows], want, ms.hidden, 1, f"prompt {i} ({lens[i]} tokens):", kind="prefill")


def test_13b_shape_prefill_of_2100_tokens_sampled_against_oracle():
    # hidden 5120, 40 x 128 heads, ffn 13824, one layer; a 2000-token prompt and a 100-token prompt in one call: every projection
    # on the 256 x 256 tile at other contraction lengths and tile counts than the 7B shape (20 / 60 / 108 weight tiles, nine
    # rows of token tiles with a ragged last one).  The oracle recomputes the short prompt (the last rows of the call) and
    # the first 64 tokens of the long one, which causal attention makes independent of the rest.
    ms = synth.WORKLOADS["C4"].shape
    seed, lens = 23, np.array([2000, 100], dtype=np.int32)
    T = int(lens.sum())
    table, nblk = synth.block_table(lens, 16, seed)
    w = make_weights(ms, seed, 1, want_f32=False)
    hidden_bits = synth.hidden_states(T, ms.hidden, seed)
    stage = make_stage(ms, w, 0, 1)
    pool = torch.zeros((1, nblk, 2, ms.n_kv_heads, 16, ms.head_dim), dtype=torch.int16, device="cuda")
    cache = binding.KVCache(pool, 0, 1, dev_i32(table))
    cu = synth.cu_seqlens(lens)
    y = stage.forward(cache, dev_i32(cu), dev_i32(np.zeros(2)), dev_bf16(hidden_bits), int(lens.max()), min_q_len=int(lens.min()))
    torch.cuda.synchronize()
    got = host_f64(y)
    assert np.isfinite(got).all()
    osh = oracle_shape(ms)
    wf = [{k: synth.bf16_bits_to_f32(v) for k, v in lw.items()} for lw in w.bits]
    for i, n in ((1, 100), (0, 64)):
        nb = (n + 15) // 16
        sub_pool = np.zeros((1, nb, 2, ms.n_kv_heads, 16, ms.head_dim), dtype=np.float32)
        rows = slice(int(cu[i]), int(cu[i]) + n)
        want = oracle.stage_forward(osh, wf, sub_pool, [0, n], [0], np.arange(nb, dtype=np.int32)[None, :],
                                    synth.bf16_bits_to_f32(hidden_bits[rows]).astype(np.float64))
        check_wide_output(got[rows], want, ms.hidden, 1, f"13B prompt {i}, first {n} tokens:", kind="prefill")


def test_full_size_prefill_workload_full_depth_sampled_against_oracle():
    # the prefill workload of the benchmark at its full size and depth (16 prompts, 15,928 tokens, 7B shape, 4 layers):
    # 128-row attention tiles, tiled projections over 125 row tiles with a ragged last one.  Attention is causal and
    # prompts are independent, so the oracle recomputes two prompts alone, whole: the shortest (420 tokens) and one above
    # 1024 tokens (1065: rows deep inside a long prompt, several 128-row tiles, a ragged last tile).
    wl = synth.WORKLOADS["C3"]
    ms, L = wl.shape, wl.n_layers
    lens = synth.draw_lengths(wl.length_dist, wl.num_seqs, wl.seed)
    T, B = int(lens.sum()), wl.num_seqs
    table, nblk = synth.block_table(lens, 16, wl.seed)
    w = make_weights(ms, wl.seed, L, want_f32=False)
    hidden_bits = synth.hidden_states(T, ms.hidden, wl.seed)
    stage = make_stage(ms, w, 0, L)
    pool = torch.zeros((L, nblk, 2, ms.n_kv_heads, 16, ms.head_dim), dtype=torch.int16, device="cuda")
    cache = binding.KVCache(pool, 0, L, dev_i32(table))
    cu = synth.cu_seqlens(lens)
    y = stage.forward(cache, dev_i32(cu), dev_i32(np.zeros(B)), dev_bf16(hidden_bits), int(lens.max()), min_q_len=int(lens.min()))
    torch.cuda.synchronize()
    got = host_f64(y)
    assert np.isfinite(got).all()
    osh = oracle_shape(ms)
    wf = [{k: synth.bf16_bits_to_f32(v) for k, v in lw.items()} for lw in w.bits]
    long_ones = [i for i in range(B) if lens[i] >= 1024]
    picks = [int(np.argmin(lens)), min(long_ones, key=lambda i: lens[i])]
    for i in picks:
        n = int(lens[i])
        nb = (n + 15) // 16
        print(f"C3: oracle on prompt {i} ({n} tokens, {L} layers)", flush=True)
        sub_pool = np.zeros((L, nb, 2, ms.n_kv_heads, 16, ms.head_dim), dtype=np.float32)
        rows = slice(int(cu[i]), int(cu[i + 1]))
        want = oracle.stage_forward(osh, wf, sub_pool, [0, n], [0], np.arange(nb, dtype=np.int32)[None, :],
                                    synth.bf16_bits_to_f32(hidden_bits[rows]).astype(np.float64))
        check_wide_output(got[rows], want, ms.hidden, L, f"prompt {i}, all {n} tokens:", kind="prefill")
        check_wide_output(got[rows][-128:], want[-128:], ms.hidden, L, f"prompt {i}, last 128 rows:", kind="prefill")
        # the cache the prompt left behind: every K and V row against the oracle's
        g_pool = synth.bf16_bits_to_f32(host_bits(cache.pool[:, cache.block_table[i, :nb].long()])).astype(np.float64)
        for l in range(L):
            g_rows = np.moveaxis(g_pool[l], 3, 1).reshape(nb * 16, -1)[:n]        # [block][kv][head][slot][D] -> token rows
            o_rows = np.moveaxis(sub_pool[l].astype(np.float64), 3, 1).reshape(nb * 16, -1)[:n]
            l2 = np.sqrt(((g_rows - o_rows) ** 2).sum(axis=1) / (o_rows ** 2).sum(axis=1))
            assert l2.max() <= 2e-2, f"prompt {i} layer {l} cache rows"
