"""The pieces of an inflight refactoring that run around the two kernels, on the GPU:

* Section 6.3: the cache transfer runs while inference continues on the old configuration --
  a snapshot pass on a second stream while decode steps append on the first, then a delta pass
  over what was appended meanwhile; the destination must hold what one pass at the end holds.
* Section 6.1, Eq. 4: the granularity score fed with stage times MEASURED through
  fxp_stage_forward at several stage depths, against the oracle's formula on the same numbers.
* Section 5 / Table 2 "Load": a stage whose parameters come from pinned host memory behaves
  exactly like one created from device-resident tensors."""
import json

import numpy as np
import pytest
import torch

import oracle
from oracle import KVView, control
from paper_2510_11938_amd import binding, granularity_profile, synth

from gpu_util import (dev_bf16, dev_i32, filled_pool_bits, host_bits, host_f64, make_stage, make_weights, oracle_shape, pool_f32,
                      rel_err)

pytestmark = pytest.mark.gpu

MID = synth.ModelShape(hidden=512, n_q_heads=8, n_kv_heads=8, head_dim=128, ffn=1024)


def test_snapshot_on_a_second_stream_while_decode_appends_then_delta_pass_equals_one_pass_at_the_end():
    ms, L, seed, steps = MID, 2, 41, 5
    osh = oracle_shape(ms)
    ctx = np.array([1500, 37, 2047, 640, 16, 999, 3000, 15], dtype=np.int32)
    B = len(ctx)
    now = ctx + steps
    w = make_weights(ms, seed, L)
    stage = make_stage(ms, w, 0, L)
    table, nblk = synth.block_table(now, 16, seed)                          # room for the tokens the steps append
    src_bits = filled_pool_bits(ms, seed, L, ctx, table, nblk)
    src = binding.KVCache(torch.from_numpy(src_bits.view(np.int16)).cuda(), 0, L, dev_i32(table))
    hidden_bits = [synth.hidden_states(B, ms.hidden, seed, salt=s) for s in range(steps)]
    xs = [dev_bf16(h) for h in hidden_bits]
    # destination: the stage re-split into [0,1) + [1,2), fresh permuted tables, pools pre-filled with a pattern
    dst_tables = [synth.block_table(now, 16, seed, salt=3 + s, spare_blocks=2) for s in range(2)]

    def fresh_dst():
        return [binding.KVCache(torch.full((1, n, 2, ms.n_kv_heads, 16, ms.head_dim), 0x3333, dtype=torch.int16, device="cuda"),
                                s, s + 1, dev_i32(t)) for s, (t, n) in enumerate(dst_tables)]

    dst = fresh_dst()
    snap_lens, cu = dev_i32(ctx), dev_i32(np.arange(B + 1))
    zero = dev_i32(np.zeros(B))
    torch.cuda.synchronize()
    side, main = torch.cuda.Stream(), torch.cuda.current_stream()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    lens_dev = [dev_i32(ctx + s) for s in range(steps + 1)]
    side.wait_stream(main)                                                  # inputs are ready; from here on the streams run free
    ev[2].record()
    stage.forward(src, cu, lens_dev[0], xs[0], 1)                           # the old configuration is decoding ...
    with torch.cuda.stream(side):                                           # ... when the snapshot starts: tokens [0, ctx)
        ev[0].record()
        binding.kv_repartition_range(ms, [src], dst, zero, snap_lens)
        ev[1].record()
    for s in range(1, steps):                                               # ... and keeps decoding while it runs
        stage.forward(src, cu, lens_dev[s], xs[s], 1)
    ev[3].record()
    main.wait_stream(side)
    binding.kv_repartition_range(ms, [src], dst, snap_lens, lens_dev[steps])  # the delta: tokens [ctx, ctx + steps)
    torch.cuda.synchronize()
    overlap = min(ev[1].elapsed_time(ev[3]), ev[2].elapsed_time(ev[1]))     # > 0 when the two ran side by side
    print(f"snapshot {ev[0].elapsed_time(ev[1]) * 1e3:.0f} us, {steps} decode steps {ev[2].elapsed_time(ev[3]) * 1e3:.0f} us, overlap {overlap * 1e3:.0f} us")

    # (1) equal to ONE pass at the end over the same source (sequential, on one stream)
    one = fresh_dst()
    binding.kv_repartition(ms, [src], one, lens_dev[steps])
    torch.cuda.synchronize()
    for a, b in zip(dst, one):
        assert torch.equal(a.pool, b.pool)
    # (2) the snapshot tokens against the oracle: its repartition of the original cache bits at the snapshot lengths
    exp = [np.full((1, n, 2, ms.n_kv_heads, 16, ms.head_dim), 0x3333, dtype=np.uint16) for _, n in dst_tables]
    oracle.kv_repartition(osh, [KVView(src_bits, 0, L, table)], [KVView(e, s, s + 1, t) for s, (e, (t, _)) in enumerate(zip(exp, dst_tables))], ctx)
    # (3) the appended tokens against the oracle: its own decode steps on its own (float) cache
    o_pool = pool_f32(src_bits)
    for s in range(steps):
        oracle.stage_forward(osh, w.f32, o_pool, np.arange(B + 1), ctx + s, table, synth.bf16_bits_to_f32(hidden_bits[s]).astype(np.float64))
    for s, (d, (t, n)) in enumerate(zip(dst, dst_tables)):
        got = host_bits(d.pool)
        got_f = synth.bf16_bits_to_f32(got).astype(np.float64)
        owned = np.zeros(n, dtype=bool)
        for i in range(B):
            for p in range(int(now[i])):
                blk, slot = t[i, p // 16], p % 16
                owned[blk] = True
                if p < ctx[i]:                                              # snapshot token: bit-exact
                    assert np.array_equal(got[0, blk, :, :, slot, :], exp[s][0, blk, :, :, slot, :]), (s, i, p)
                else:                                                       # appended meanwhile: the oracle's row, to the stage tolerance
                    o = o_pool[s, table[i, p // 16], :, :, slot, :].astype(np.float64).reshape(-1, ms.head_dim)
                    assert rel_err(got_f[0, blk, :, :, slot, :].reshape(-1, ms.head_dim), o) <= 2e-2, (s, i, p)
            tail = int(now[i]) % 16
            if tail:                                                        # slots after the last valid token arrive as zero
                assert not got[0, t[i, (int(now[i]) - 1) // 16], :, :, tail:, :].any()
        assert (got[0, ~owned] == 0x3333).all()                             # blocks no sequence maps to are not written


def test_granularity_scores_from_measured_stage_times_match_the_oracle_formula():
    # Table-2 analogue: one decode step of a 7B-shaped stage of 1 and 2 layers, timed through fxp_stage_forward
    ms, layers_total, batch = synth.LLAMA2_7B, 32, 8
    ctx = synth.draw_lengths(("uniform", 256, 1024), batch, seed=1)
    handoff_ms = 0.012
    times = {d: granularity_profile.measure_stage_ms(ms, d, batch, ctx, steps=10) for d in (1, 2)}
    print("measured stage times (ms):", times)
    assert 0.02 < times[1] < times[2] < 20.0                                # real, and deeper costs more
    assert 1.5 <= times[2] / times[1] <= 2.5                                # compute is about linear in depth
    cands = [granularity_profile.stage_candidate(layers_total, d, batch, times[d], handoff_ms) for d in (1, 2)]
    cvs = [0.5, 1.0, 2.0, 4.0]
    granularity_profile.spread_cv_opt(cands, cvs)
    T = [batch / ((times[d] + handoff_ms) * 1e-3) for d in (1, 2)]          # restated here from the measured times
    Lk = [layers_total // d * (times[d] + handoff_ms) for d in (1, 2)]
    assert [c.n_stages for c in cands] == [32, 16]
    np.testing.assert_allclose([c.throughput for c in cands], T, rtol=1e-12)
    np.testing.assert_allclose([c.latency for c in cands], Lk, rtol=1e-12)
    nu = [c.cv_opt for c in cands]
    for alpha, sigma in ((0.5, 1.0), (0.9, 0.3), (0.0, 2.0)):
        picks = granularity_profile.select_for_cvs(cands, cvs, alpha, sigma)
        for pk in picks:
            want = control.granularity_scores(T, Lk, nu, pk["cv"], alpha, sigma)
            np.testing.assert_allclose(pk["scores"], want, rtol=1e-12)
            assert pk["selected_n_stages"] == cands[control.select_granularity(T, Lk, nu, pk["cv"], alpha, sigma)].n_stages


def test_granularity_profile_command_end_to_end(capsys):
    # the script as a user runs it (7B shape, two depths, with the load column): its JSON is consistent with the oracle
    rc = granularity_profile.main(["--depths", "1,2", "--batch", "4", "--ctx", "64,256", "--steps", "5", "--load", "--cvs", "0.5,3"])
    assert rc == 0
    rep = json.loads(capsys.readouterr().out.strip().splitlines()[-1])
    rows = rep["stages"]
    assert [r["layers_per_stage"] for r in rows] == [1, 2] and all(r["compute_ms"] > 0 for r in rows)
    for r in rows:
        assert r["load"]["bytes"] == synth.LLAMA2_7B.params_per_layer * 2 * r["layers_per_stage"]
        assert r["load"]["h2d_ms"] > 0 and r["load"]["retile_ms"] > 0
    T = [r["throughput_tokens_s"] for r in rows]
    Lk = [r["latency_ms"] for r in rows]
    for pk in rep["picks"]:
        want = control.granularity_scores(T, Lk, rep["cv_opt"], pk["cv"], rep["alpha"], rep["sigma"])
        np.testing.assert_allclose(pk["scores"], want, rtol=1e-9)
        assert pk["selected_n_stages"] == rows[int(np.argmax(want))]["n_stages"]


def test_stage_loaded_from_pinned_host_memory_equals_a_stage_created_from_device_tensors():
    ms, L, seed = MID, 3, 43
    w = make_weights(ms, seed, L)
    host_layers = [{k: torch.from_numpy(v.view(np.int16)).view(torch.bfloat16).pin_memory() for k, v in lw.items()} for lw in w.bits]
    loaded, h2d_ms, retile_ms = granularity_profile.load_stage(ms, host_layers)
    assert h2d_ms > 0 and retile_ms > 0
    fresh = make_stage(ms, w, 0, L)
    assert torch.equal(loaded.arena, fresh.arena)                            # the same re-tiled records
    ctx, q_lens = np.array([300, 17, 1025, 64], dtype=np.int32), np.array([1, 1, 1, 1], dtype=np.int32)
    table, nblk = synth.block_table(ctx + 1, 16, seed)
    bits = filled_pool_bits(ms, seed, L, ctx, table, nblk)
    x = dev_bf16(synth.hidden_states(4, ms.hidden, seed))
    outs = []
    for st in (loaded, fresh):
        cache = binding.KVCache(torch.from_numpy(bits.view(np.int16)).cuda(), 0, L, dev_i32(table))
        outs.append(st.forward(cache, dev_i32(synth.cu_seqlens(q_lens)), dev_i32(ctx), x, 1))
    torch.cuda.synchronize()
    assert torch.equal(outs[0].view(torch.int16), outs[1].view(torch.int16))
    want = oracle.stage_forward(oracle_shape(ms), w.f32, pool_f32(bits), synth.cu_seqlens(q_lens), ctx, table,
                                synth.bf16_bits_to_f32(synth.hidden_states(4, ms.hidden, seed)).astype(np.float64))
    assert rel_err(host_f64(outs[0]), want) <= 2e-2
