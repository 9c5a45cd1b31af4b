"""Pins for the oracle's stage forward: an independent dense float64
re-statement, and the invariants the paper fixes for a pipeline stage:
  (1) stages are a disjoint cover of the graph (Section 5, Eq. 2 constraints)
      => composing split stages equals the unsplit stage;
  (2) the KV cache must stay consistent (Section 6.3)
      => cached incremental decode equals recomputing the whole prefix;
  (4) refactoring happens without service interruption (Section 6)
      => a step after KV repartition equals the same step without it."""
import numpy as np
import pytest
import torch

import oracle
from oracle import KVView, Shape
from paper_2510_11938_amd import synth

from dense_ref import DenseStage

TINY = synth.TINY
SH = Shape(TINY.hidden, TINY.n_q_heads, TINY.n_kv_heads, TINY.head_dim, TINY.ffn,
           TINY.kv_block_size, TINY.rms_eps, TINY.rope_base)
GQA = Shape(hidden=128, n_q_heads=8, n_kv_heads=2, head_dim=16, ffn=176, kv_block_size=16)


def weights_f32(shape, seed, n_layers):
    ms = synth.ModelShape(shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.ffn,
                          shape.rms_eps, shape.rope_base, shape.kv_block_size)
    return [{k: synth.bf16_bits_to_f32(v) for k, v in synth.layer_weights(ms, seed, l).items()}
            for l in range(n_layers)]


def hidden_f64(T, H, seed, salt=0):
    return synth.bf16_bits_to_f32(synth.hidden_states(T, H, seed, salt)).astype(np.float64)


@pytest.mark.parametrize("shape", [SH, GQA], ids=["tiny-mha", "gqa"])
def test_prefill_then_decode_matches_dense_float64_restatement(shape):
    L = 2
    W = weights_f32(shape, 0, L)
    lens = np.array([19, 33, 5, 16], dtype=np.int32)
    table, nblk = synth.block_table(lens + 2, shape.kv_block_size, seed=0)
    pool = oracle.new_pool(shape, L, nblk)
    dense = DenseStage(shape, W)
    ids = list(range(len(lens)))
    # prefill of whole prompts
    x = hidden_f64(int(lens.sum()), shape.hidden, 0)
    y = oracle.stage_forward(shape, W, pool, synth.cu_seqlens(lens), np.zeros_like(lens), table, x)
    yd = dense.forward(ids, lens.tolist(), [0] * len(lens), torch.from_numpy(x)).numpy()
    # keys and values are read back from the oracle's float32 cache, hence ~1e-7, not 1e-15
    assert np.abs(y - yd).max() < 2e-6
    # two decode steps on top of the cache the prefill wrote (the oracle's cache is float storage)
    ctx = lens.copy()
    for step in range(2):
        x = hidden_f64(len(lens), shape.hidden, 0, salt=1 + step)
        y = oracle.stage_forward(shape, W, pool, np.arange(len(lens) + 1), ctx, table, x)
        yd = dense.forward(ids, [1] * len(lens), ctx.tolist(), torch.from_numpy(x)).numpy()
        assert np.abs(y - yd).max() < 2e-6
        ctx += 1


def test_attention_probabilities_rows_sum_to_one_and_are_causal():
    W = weights_f32(SH, 0, 1)
    lens = np.array([7, 21], dtype=np.int32)
    table, nblk = synth.block_table(lens, SH.kv_block_size, seed=3)
    pool = oracle.new_pool(SH, 1, nblk)
    x = hidden_f64(int(lens.sum()), SH.hidden, 3)
    _, probs = oracle.stage_forward(SH, W, pool, synth.cu_seqlens(lens), [0, 0], table, x, probs_stride=21)
    at = 0
    for n in lens:
        for j in range(n):
            row = probs[0, at + j]
            assert np.allclose(row[:, : j + 1].sum(axis=1), 1.0, rtol=1e-13)
            assert np.all(row[:, j + 1:] == 0.0)
        at += n


def test_split_stages_compose_to_unsplit_stage_bit_exact():
    # Eq. 2 constraints: union of stages = all operators, stages disjoint.
    L = 2
    W = weights_f32(SH, 0, L)
    lens = synth.draw_lengths(("uniform", 32, 128), 4, seed=0)
    x = hidden_f64(int(lens.sum()), SH.hidden, 0)
    cu = synth.cu_seqlens(lens)
    zero = np.zeros_like(lens)
    # unsplit [0,2): one pool, one table
    t_all, n_all = synth.block_table(lens + 1, SH.kv_block_size, seed=0, salt=0)
    p_all = oracle.new_pool(SH, 2, n_all)
    y_all = oracle.stage_forward(SH, W, p_all, cu, zero, t_all, x)
    # split [0,1) + [1,2): separate pools and differently permuted tables
    t0, n0 = synth.block_table(lens + 1, SH.kv_block_size, seed=0, salt=1)
    t1, n1 = synth.block_table(lens + 1, SH.kv_block_size, seed=0, salt=2, spare_blocks=3)
    p0, p1 = oracle.new_pool(SH, 1, n0), oracle.new_pool(SH, 1, n1)
    mid = oracle.stage_forward(SH, W[:1], p0, cu, zero, t0, x)
    y_split = oracle.stage_forward(SH, W[1:], p1, cu, zero, t1, mid)
    assert np.array_equal(y_all, y_split)
    # decode step on top: still identical
    xd = hidden_f64(len(lens), SH.hidden, 0, salt=9)
    cud = np.arange(len(lens) + 1)
    yd_all = oracle.stage_forward(SH, W, p_all, cud, lens, t_all, xd)
    yd_split = oracle.stage_forward(SH, W[1:], p1, cud, lens, t1,
                                    oracle.stage_forward(SH, W[:1], p0, cud, lens, t0, xd))
    assert np.array_equal(yd_all, yd_split)


def test_cached_decode_equals_full_recompute_and_chunked_prefill_equals_one_shot():
    L = 2
    W = weights_f32(SH, 0, L)
    lens = np.array([40, 17, 64], dtype=np.int32)
    T = int(lens.sum())
    x_full = hidden_f64(T + len(lens), SH.hidden, 5)          # rows for n+1 tokens per sequence
    # split the rows: first n_i rows of sequence i are the prompt, the last is the decode token
    cu1 = synth.cu_seqlens(lens + 1)
    prompt_rows = np.concatenate([np.arange(cu1[i], cu1[i] + lens[i]) for i in range(len(lens))])
    last_rows = cu1[1:] - 1
    table, nblk = synth.block_table(lens + 1, SH.kv_block_size, seed=5)
    # (a) one shot over n+1 tokens
    pa = oracle.new_pool(SH, L, nblk)
    ya = oracle.stage_forward(SH, W, pa, cu1, np.zeros_like(lens), table, x_full)
    # (b) prefill n, then decode 1 with the cache
    pb = oracle.new_pool(SH, L, nblk)
    yb_pre = oracle.stage_forward(SH, W, pb, synth.cu_seqlens(lens), np.zeros_like(lens), table, x_full[prompt_rows])
    yb_dec = oracle.stage_forward(SH, W, pb, np.arange(len(lens) + 1), lens, table, x_full[last_rows])
    assert np.abs(yb_dec - ya[last_rows]).max() < 2e-6          # float cache storage is the only difference
    assert np.abs(yb_pre - ya[prompt_rows]).max() < 2e-6
    # (c) chunked prefill: chunks of at most 16 tokens per sequence per call
    pc = oracle.new_pool(SH, L, nblk)
    done = np.zeros_like(lens)
    yc = np.zeros_like(ya)
    while np.any(done < lens + 1):
        take = np.minimum(16, lens + 1 - done)
        rows = np.concatenate([np.arange(cu1[i] + done[i], cu1[i] + done[i] + take[i]) for i in range(len(lens))])
        yc[rows] = oracle.stage_forward(SH, W, pc, synth.cu_seqlens(take), done, table, x_full[rows])
        done = done + take
    assert np.abs(yc - ya).max() < 2e-6
    assert np.abs(pc - pa).max() < 1e-6


def test_output_invariant_under_physical_block_permutation():
    W = weights_f32(SH, 1, 1)
    lens = np.array([33, 50], dtype=np.int32)
    x = hidden_f64(int(lens.sum()), SH.hidden, 6)
    outs = []
    for salt in (0, 1):
        table, nblk = synth.block_table(lens, SH.kv_block_size, seed=6, salt=salt, spare_blocks=salt * 5)
        pool = oracle.new_pool(SH, 1, nblk)
        outs.append(oracle.stage_forward(SH, W, pool, synth.cu_seqlens(lens), [0, 0], table, x))
    assert np.array_equal(outs[0], outs[1])


def test_decode_after_merge_repartition_equals_decode_on_split_stages():
    # Serving continues unchanged across a refactor: split stages [0,1)+[1,2) hold the cache,
    # it is merged into a fresh [0,2) pool, and the next decode step gives identical output.
    L = 2
    W = weights_f32(SH, 0, L)
    lens = synth.draw_lengths(("uniform", 32, 128), 4, seed=0)
    cu = synth.cu_seqlens(lens)
    x = hidden_f64(int(lens.sum()), SH.hidden, 0)
    t0, n0 = synth.block_table(lens + 1, SH.kv_block_size, seed=0, salt=1)
    t1, n1 = synth.block_table(lens + 1, SH.kv_block_size, seed=0, salt=2)
    p0, p1 = oracle.new_pool(SH, 1, n0), oracle.new_pool(SH, 1, n1)
    zero = np.zeros_like(lens)
    oracle.stage_forward(SH, W[1:], p1, cu, zero, t1, oracle.stage_forward(SH, W[:1], p0, cu, zero, t0, x))
    # merge
    tm, nm = synth.block_table(lens + 1, SH.kv_block_size, seed=0, salt=3, spare_blocks=2)
    pm = oracle.new_pool(SH, 2, nm)
    oracle.kv_repartition(SH, [KVView(p0, 0, 1, t0), KVView(p1, 1, 2, t1)], [KVView(pm, 0, 2, tm)], lens)
    xd = hidden_f64(len(lens), SH.hidden, 0, salt=9)
    cud = np.arange(len(lens) + 1)
    y_split = oracle.stage_forward(SH, W[1:], p1, cud, lens, t1,
                                   oracle.stage_forward(SH, W[:1], p0, cud, lens, t0, xd))
    y_merged = oracle.stage_forward(SH, W, pm, cud, lens, tm, xd)
    assert np.array_equal(y_split, y_merged)
