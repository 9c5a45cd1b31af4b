"""Writes the stored expected values under tests/golden/ from the oracle alone.

    python tests/golden/make_golden.py

The paper prints no worked numeric example of a stage step or of a cache migration (its only
numbers on this path are Table 2's timings), so these fixtures are not the paper's values: they
freeze what the pinned oracle computes on the tiny configuration, so that a later change to the
oracle's arithmetic cannot pass unnoticed.  Nothing here touches the GPU library.
"""
import hashlib
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle                                   # noqa: E402
from oracle import KVView, Shape                # noqa: E402
from paper_2510_11938_amd import synth          # noqa: E402


def tiny_inputs():
    """C1: two layers of the tiny shape as stages [0,1) + [1,2), four sequences, a cache of synthetic rows
    per stage (each with its own permuted block table), one row of hidden state per sequence."""
    wl = synth.WORKLOADS["C1"]
    ms = wl.shape
    ctx = synth.draw_lengths(wl.length_dist, wl.num_seqs, wl.seed)
    w_bits = [synth.layer_weights(ms, wl.seed, l) for l in range(2)]
    x_bits = synth.hidden_states(wl.num_seqs, ms.hidden, wl.seed)
    views = []
    for l in range(2):
        table, nblk = synth.block_table(ctx + 1, 16, wl.seed, salt=l)
        pool = np.zeros((1, nblk, 2, ms.n_kv_heads, 16, ms.head_dim), dtype=np.uint16)
        for i in range(wl.num_seqs):
            synth.fill_pool_rows(pool, 0, table[i], synth.cache_rows(ms, wl.seed, i, l, int(ctx[i])), 16)
        views.append((pool, table))
    t2, n2 = synth.block_table(ctx + 1, 16, wl.seed, salt=7)
    return ms, ctx, w_bits, x_bits, views, (t2, n2)


def tiny_case():
    """One decode step through the two stages, then the merge of the two caches (as they were before the
    step: the tokens valid in ctx) into one stage [0,2) with a fresh table over a 0xABCD-filled pool."""
    ms, ctx, w_bits, x_bits, views, (t2, n2) = tiny_inputs()
    sh = Shape(ms.hidden, ms.n_q_heads, ms.n_kv_heads, ms.head_dim, ms.ffn, ms.kv_block_size, ms.rms_eps, ms.rope_base)
    W = [{k: synth.bf16_bits_to_f32(v) for k, v in lw.items()} for lw in w_bits]
    x = synth.bf16_bits_to_f32(x_bits).astype(np.float64)
    cu = np.arange(len(ctx) + 1)
    src = [KVView(views[0][0].copy(), 0, 1, views[0][1]), KVView(views[1][0].copy(), 1, 2, views[1][1])]
    dst = [KVView(np.full((2, n2, 2, ms.n_kv_heads, 16, ms.head_dim), 0xABCD, dtype=np.uint16), 0, 2, t2)]
    oracle.kv_repartition(sh, src, dst, ctx)
    p0 = synth.bf16_bits_to_f32(views[0][0]); p1 = synth.bf16_bits_to_f32(views[1][0])
    mid = oracle.stage_forward(sh, W[:1], p0, cu, ctx, views[0][1], x)
    out = oracle.stage_forward(sh, W[1:], p1, cu, ctx, views[1][1], mid)
    return ctx, out, dst[0].pool


def main():
    ctx, out, merged = tiny_case()
    with open(os.path.join(HERE, "c1_decode_and_merge.txt"), "w") as f:
        f.write("# oracle, workload C1 (tiny shape, stages [0,1)+[1,2), seed 0): written by tests/golden/make_golden.py\n")
        f.write("# not values from the paper (it prints none for this path); a freeze of the pinned oracle\n")
        f.write("ctx_lens " + " ".join(str(int(c)) for c in ctx) + "\n")
        for i in range(out.shape[0]):
            for k in range(0, out.shape[1], 37):            # every 37th column of every output row
                f.write(f"hidden_out {i} {k} {float(out[i, k])!r}\n")
        for i in range(out.shape[0]):
            f.write(f"row_rms {i} {float(np.sqrt((out[i] ** 2).mean()))!r}\n")
        f.write(f"hidden_out_sum {float(out.sum())!r}\n")
        f.write(f"hidden_out_abs_sum {float(np.abs(out).sum())!r}\n")
        f.write("merged_pool_sha256 " + hashlib.sha256(np.ascontiguousarray(merged).tobytes()).hexdigest() + "\n")
    print("wrote", os.path.join(HERE, "c1_decode_and_merge.txt"))


if __name__ == "__main__":
    main()
