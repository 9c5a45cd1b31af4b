"""Full-width parity cases for the larger workload shapes: the GPU runs the whole
batch at the real head geometry and widths (13B MHA 40x128, 70B GQA 64/8x128),
the oracle recomputes sampled sequences one by one (batch rows are independent)
from the same bits.  Layer counts are cut to keep the host-side generation
short; every layer runs the same kernels at the same shapes."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_11938_amd import binding, synth

from gpu_util import (check_wide_output, dev_bf16, dev_i32, filled_pool_bits, host_f64, make_stage, make_weights,
                      oracle_shape, pool_f32)

pytestmark = pytest.mark.gpu


def run_sampled_decode(wl_name, n_layers, samples):
    wl = synth.WORKLOADS[wl_name]
    ms = wl.shape
    ctx = synth.draw_lengths(wl.length_dist, wl.num_seqs, wl.seed)
    table, nblk = synth.block_table(ctx + 1, 16, wl.seed)
    w = make_weights(ms, wl.seed, n_layers, want_f32=False)
    pool_bits = filled_pool_bits(ms, wl.seed, n_layers, ctx, table, nblk, threads=16)
    hidden_bits = synth.hidden_states(wl.num_seqs, ms.hidden, wl.seed)
    stage = make_stage(ms, w, 0, n_layers)
    cache = binding.KVCache(torch.from_numpy(pool_bits.view(np.int16)).cuda(), 0, n_layers, dev_i32(table))
    y = stage.forward(cache, dev_i32(np.arange(wl.num_seqs + 1)), dev_i32(ctx), dev_bf16(hidden_bits), 1)
    torch.cuda.synchronize()
    got = host_f64(y)
    assert np.isfinite(got).all()
    osh = oracle_shape(ms)
    wf = [{k: synth.bf16_bits_to_f32(v) for k, v in lw.items()} for lw in w.bits]
    picks = [int(np.argmin(ctx)), int(np.argmax(ctx))] + list(samples)
    for i in picks:
        nb = (int(ctx[i]) + 16) // 16
        sub_pool = pool_f32(pool_bits[:, table[i, :nb]])
        want = oracle.stage_forward(osh, wf, sub_pool, [0, 1], [ctx[i]], np.arange(nb, dtype=np.int32)[None, :],
                                    synth.bf16_bits_to_f32(hidden_bits[i:i + 1]).astype(np.float64))
        check_wide_output(got[i:i + 1], want, f"{wl_name} sequence {i} ctx {ctx[i]}:")
    return ms, ctx, cache, table


def test_70b_gqa_shape_decode_batch_128_sampled_against_oracle():
    # hidden 8192, 64 query / 8 kv heads x 128, ffn 28672, batch 128, contexts U[1024,8192]; 1 layer
    run_sampled_decode("C5", 1, samples=[17])


def test_13b_shape_decode_batch_64_then_resplit_sampled_against_oracle():
    # hidden 5120, 40 x 128 heads, ffn 13824, batch 64, lognormal contexts; 2 layers, then re-split 2 -> 1 + 1
    ms, ctx, cache, table = run_sampled_decode("C4", 2, samples=[5])
    lens = ctx + 1                                           # the step appended one token per sequence
    dst = []
    for s in range(2):
        t, n = synth.block_table(lens, 16, 3, salt=7 + s, spare_blocks=2)
        dst.append(binding.KVCache(torch.full((1, n, 2, ms.n_kv_heads, 16, ms.head_dim), 0x2222, dtype=torch.int16, device="cuda"),
                                   s, s + 1, dev_i32(t)))
    binding.kv_repartition(ms, [cache], dst, dev_i32(lens))
    torch.cuda.synchronize()
    nblk = (lens + 15) // 16
    src_pool = cache.pool.view(torch.int16)
    for s, dv in enumerate(dst):
        owned = torch.zeros(dv.pool.shape[1], dtype=torch.bool, device="cuda")
        for i in range(len(lens)):
            sb = cache.block_table[i, : nblk[i]].long(); db = dv.block_table[i, : nblk[i]].long()
            owned[db] = True
            want = src_pool[s:s + 1][:, sb].clone()
            tail = int(lens[i] % 16)
            if tail:
                want[:, -1, :, :, tail:, :] = 0
            assert torch.equal(dv.pool[:, db], want), f"stage {s} sequence {i}"
        assert bool((dv.pool[:, ~owned] == 0x2222).all())


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
        check_wide_output(got[rows], want, f"prompt {i} ({lens[i]} tokens):")


def test_full_size_prefill_workload_sampled_against_oracle():
    # the prefill workload of the benchmark at its full size (16 prompts, 15,928 tokens, 7B shape, 1 layer): 128-row
    # attention tiles, tiled projections over 125 row tiles with a ragged last one.  Attention is causal and prompts are
    # independent, so the first n output rows of a prompt are what the stage gives for its first n tokens alone: the
    # oracle recomputes three such heads of prompts (first, shortest, last in the batch).
    wl = synth.WORKLOADS["C3"]
    ms = wl.shape
    lens = synth.draw_lengths(wl.length_dist, wl.num_seqs, wl.seed)
    T, B = int(lens.sum()), wl.num_seqs
    table, nblk = synth.block_table(lens, 16, wl.seed)
    w = make_weights(ms, wl.seed, 1, want_f32=False)
    hidden_bits = synth.hidden_states(T, ms.hidden, wl.seed)
    stage = make_stage(ms, w, 0, 1)
    pool = torch.zeros((1, nblk, 2, ms.n_kv_heads, 16, ms.head_dim), dtype=torch.int16, device="cuda")
    cache = binding.KVCache(pool, 0, 1, dev_i32(table))
    cu = synth.cu_seqlens(lens)
    y = stage.forward(cache, dev_i32(cu), dev_i32(np.zeros(B)), dev_bf16(hidden_bits), int(lens.max()), min_q_len=int(lens.min()))
    torch.cuda.synchronize()
    got = host_f64(y)
    assert np.isfinite(got).all()
    osh = oracle_shape(ms)
    wf = [{k: synth.bf16_bits_to_f32(v) for k, v in lw.items()} for lw in w.bits]
    for i, n in ((0, 150), (int(np.argmin(lens)), 130), (B - 1, 100)):
        nb = (n + 15) // 16
        sub_pool = np.zeros((1, nb, 2, ms.n_kv_heads, 16, ms.head_dim), dtype=np.float32)
        rows = slice(int(cu[i]), int(cu[i]) + n)
        want = oracle.stage_forward(osh, wf, sub_pool, [0, n], [0], np.arange(nb, dtype=np.int32)[None, :],
                                    synth.bf16_bits_to_f32(hidden_bits[rows]).astype(np.float64))
        check_wide_output(got[rows], want, f"prompt {i}, first {n} of {lens[i]} tokens:")
