#!/usr/bin/env python3
"""Benchmark of the stage-forward / KV-repartition hot path on one MI355X.

One step = one decode pass of the whole stage (Llama-2-7B-shaped, 4 layers,
batch 32, contexts uniform in [512,4096], permuted block table) followed, as a
separately timed leg, by the KV repartition of that stage's cache (4 layers ->
2 + 2 into fresh permuted tables).  Inputs are synthetic, seeded, and resident
in HBM before the timed region starts.

Prints one JSON line: decode tokens/s as `value`, the repartition rate, the
roofline of the dominant kernel (paged decode attention, HBM bound) measured
with HIP events around each launch, and the CPU oracle timed on a bounded sample
of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def read_traffic(path: str, kernel: str):
    """HBM bytes per launch measured with rocprofv3 counters, if a summary was committed."""
    try:
        for line in open(path):
            if line.startswith(f"traffic_bytes_per_launch[{kernel}]:"):
                return float(line.split(":", 1)[1].split()[0])
    except OSError:
        pass
    return None


MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X published dense bf16 peak
CALIBRATION_COPY_BYTES = 1 << 30


def calibration_copy(torch, dev) -> None:
    """One plain device-to-device copy of a known size (1 GiB read + 1 GiB written).  It is not
    timed; a `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE` run of this same command reads the
    counters of this copy kernel next to those of the library's kernels, which gives the factor
    that turns counter units into bytes."""
    src = torch.empty(CALIBRATION_COPY_BYTES // 4, dtype=torch.int32, device=dev)
    src.fill_(3)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    dst.copy_(src)
    torch.cuda.synchronize()



def timed_steps(torch, step, k):
    """k steps, each between two events on the current stream, the whole loop between two synchronisations.
    Returns ([ms of each step], wall-clock ms per step over the loop)."""
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(k + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev[0].record()
    for i in range(k):
        step()
        ev[i + 1].record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / k
    return [ev[i].elapsed_time(ev[i + 1]) for i in range(k)], wall


def prefill_record(torch, wl, stage, steps, warmup, weights_note=""):
    """One step = the chunked-prefill forward of the whole ragged batch of workload ``wl`` (prompts log-uniform in
    [256,2048], empty cache) through ``stage``.  Returns the record: prefill tokens/s (median of event-timed steps) and
    the MFMA roofline of the tiled projection kernel from HIP events around each of its launches."""
    from paper_2510_11938_amd import binding, synth
    ms, L, B = wl.shape, wl.n_layers, wl.num_seqs
    dev = torch.device("cuda:0")
    lens = synth.draw_lengths(wl.length_dist, B, wl.seed)
    T = int(lens.sum())
    table, nblk = synth.block_table(lens, 16, wl.seed)
    cache = binding.KVCache(torch.zeros((L, nblk, 2, ms.n_kv_heads, 16, ms.head_dim), dtype=torch.int16, device=dev), 0, L,
                            torch.from_numpy(table).to(dev))
    x = torch.from_numpy(synth.hidden_states(T, ms.hidden, wl.seed).view(np.int16)).to(dev).view(torch.bfloat16)
    y = torch.empty_like(x)
    cu = torch.from_numpy(synth.cu_seqlens(lens)).to(dev)
    cl = torch.zeros(B, dtype=torch.int32, device=dev)
    mq = int(lens.max())

    def step():
        stage.forward(cache, cu, cl, x, mq, hidden_out=y, min_q_len=int(lens.min()))

    for _ in range(warmup):
        step()
    step_ms, wall_ms = timed_steps(torch, step, steps)
    ms_per_step = float(np.median(step_ms))
    binding.profile_enable(True)
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    prof = binding.profile_read()
    binding.profile_enable(False)
    kernels = {k: {"avg_us": v["ms"] * 1e3 / v["launches"], "launches_per_step": v["launches"] / steps} for k, v in prof.items()}
    flops_layer = 2 * T * (ms.params_per_layer - 2 * ms.hidden)          # the four projections of one layer
    gemm_ms_layer = kernels["gemm_tiled"]["avg_us"] * 4 / 1e3
    tflops = flops_layer / (gemm_ms_layer * 1e-3) / 1e12
    attn_flops_layer = 2 * 2 * int((lens.astype(np.int64) * (lens.astype(np.int64) + 1) // 2).sum()) * ms.n_q_heads * ms.head_dim
    return {
        "metric": "stage prefill tokens/s (7B shape, 4 layers, 16 ragged prompts)", "value": T / (ms_per_step * 1e-3), "unit": "tokens/s",
        "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step, "ms_per_step_wall_mean": wall_ms, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{wl.name}: {ms.hidden}-hidden {ms.n_q_heads}/{ms.n_kv_heads}x{ms.head_dim} heads, ffn {ms.ffn}, {L} layers, "
                               f"{B} prompts {wl.length_dist}, {T} tokens, kv block 16" + weights_note, "seed": wl.seed},
        "roofline": {"kernel": "gemm_wide_kernel (the projections of a step above 2047 token rows; profile class gemm_tiled)", "bound": "mfma", "achieved": tflops, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": tflops / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                     "algorithmic_flops_per_layer": flops_layer, "avg_launch_us": kernels["gemm_tiled"]["avg_us"]},
        "attn_prefill": {"avg_launch_us": kernels["attn_prefill"]["avg_us"], "causal_flops_per_layer": attn_flops_layer,
                         "TFLOPs": attn_flops_layer / (kernels["attn_prefill"]["avg_us"] * 1e-6) / 1e12},
        "kernels": kernels,
    }


def bench_prefill(args, wl) -> int:
    """Secondary mode (--workload C3): the prefill step as the headline of its own JSON line."""
    import torch
    from paper_2510_11938_amd import binding, synth
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    ms, L = wl.shape, wl.n_layers
    w_dev = [{k: torch.from_numpy(np.ascontiguousarray(v).view(np.int16)).to(dev).view(torch.bfloat16)
              for k, v in synth.layer_weights(ms, wl.seed, l).items()} for l in range(L)]
    stage = binding.Stage(ms, 0, L, w_dev)
    torch.cuda.synchronize()
    del w_dev
    out = prefill_record(torch, wl, stage, args.steps, args.warmup)
    out.update({"n_gpus": 1, "higher_is_better": True, "scaling": "weak", "vs_baseline": None})
    calibration_copy(torch, dev)
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps (default 50 for decode, 5 for prefill)")
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="C2", help="synthetic workload id (C2 is the headline configuration)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-prefill", action="store_true", help="skip the chunked-prefill sub-record (workload C3 through the same stage)")
    ap.add_argument("--no-incremental", action="store_true",
                    help="skip the concurrent-snapshot / delta-pass leg (keeps a kernel trace free of deliberately overlapped kernels)")
    ap.add_argument("--cpu-sample-seqs", type=int, default=0, help="sequences the oracle is timed on (0 = the whole batch)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus must be 1", file=sys.stderr)
        return 2

    import torch
    from concurrent.futures import ThreadPoolExecutor
    from paper_2510_11938_amd import binding, synth

    wl = synth.WORKLOADS[args.workload]
    if args.steps is None:
        args.steps = 50 if wl.kind == "decode" else 5
    if args.warmup is None:
        args.warmup = 10 if wl.kind == "decode" else 2
    if wl.kind == "prefill":
        return bench_prefill(args, wl)
    ms, L, B = wl.shape, wl.n_layers, wl.num_seqs
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    def to_dev(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(dev).view(torch.bfloat16)

    # ---- inputs (seeded, synthetic) -------------------------------------------------
    t_setup = time.time()
    ctx = synth.draw_lengths(wl.length_dist, B, wl.seed)
    table, nblk = synth.block_table(ctx + 1, 16, wl.seed)
    with ThreadPoolExecutor(max_workers=8) as ex:        # every layer has a generator of its own
        w_bits = list(ex.map(lambda l: synth.layer_weights(ms, wl.seed, l), range(L)))
    w_dev = [{k: to_dev(v) for k, v in lw.items()} for lw in w_bits]
    stage = binding.Stage(ms, 0, L, w_dev)
    torch.cuda.synchronize()
    del w_dev                                            # the stage keeps its own re-tiled copy
    pool_host = np.zeros((L, nblk, 2, ms.n_kv_heads, 16, ms.head_dim), dtype=np.uint16)

    def fill(job):
        i, l = job
        synth.fill_pool_rows(pool_host, l, table[i], synth.cache_rows(ms, wl.seed, i, l, int(ctx[i])), 16)

    with ThreadPoolExecutor(max_workers=16) as ex:
        list(ex.map(fill, [(i, l) for i in range(B) for l in range(L)]))
    cache = binding.KVCache(torch.from_numpy(pool_host.view(np.int16)).to(dev), 0, L,
                            torch.from_numpy(table).to(dev))
    hidden_bits = synth.hidden_states(B, ms.hidden, wl.seed)
    x = to_dev(hidden_bits)
    y = torch.empty_like(x)
    cu = torch.arange(B + 1, dtype=torch.int32, device=dev)
    cl = torch.from_numpy(ctx).to(dev)
    setup_s = time.time() - t_setup

    def step():
        stage.forward(cache, cu, cl, x, 1, hidden_out=y)

    # ---- decode: W warm-up steps, then exactly K timed steps -------------------------
    # Every step is bracketed by HIP events on the stream the library launches on; `value` is the median step, the
    # wall-clock mean over the same K steps and the very first step of the process are reported beside it.
    first_ms = timed_steps(torch, step, 1)[0][0]
    for _ in range(max(0, args.warmup - 1)):
        step()
    step_ms, wall_ms = timed_steps(torch, step, args.steps)
    ms_per_step = float(np.median(step_ms))
    tokens_per_s = B / (ms_per_step * 1e-3)

    # ---- per-kernel durations: the same K steps again with an event pair around each launch
    binding.profile_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    prof = binding.profile_read()
    binding.profile_enable(False)

    n_keys = int((ctx.astype(np.int64) + 1).sum())
    kv_bytes_per_token = 2 * ms.n_kv_heads * ms.head_dim * 2
    attn_bytes = n_keys * kv_bytes_per_token                         # per launch = per layer
    weight_bytes_layer = 2 * (ms.params_per_layer - 2 * ms.hidden)   # the four projections of one layer
    kernels = {}
    for name, rec in prof.items():
        kernels[name] = {"avg_us": rec["ms"] * 1e3 / rec["launches"], "launches_per_step": rec["launches"] / args.steps}
    attn_us = kernels["attn_decode"]["avg_us"]
    attn_gbps = attn_bytes / (attn_us * 1e-6) / 1e9
    skinny_us_layer = kernels["gemm_skinny"]["avg_us"] * 4
    kernels["attn_decode"]["GBps"] = attn_gbps
    kernels["gemm_skinny"]["weight_stream_GBps"] = weight_bytes_layer / (skinny_us_layer * 1e-6) / 1e9
    ideal_ms = (L * weight_bytes_layer + L * attn_bytes) / (HBM_PEAK_GBPS * 1e9) * 1e3

    # ---- KV repartition: the stage's cache re-split 4 -> 2 + 2 into fresh tables -------
    half = L // 2
    dst = []
    for s, (a, b) in enumerate([(0, half), (half, L)]):
        t, n = synth.block_table(ctx + 1, 16, wl.seed, salt=1 + s)
        dst.append(binding.KVCache(torch.zeros((b - a, n, 2, ms.n_kv_heads, 16, ms.head_dim), dtype=torch.int16, device=dev),
                                   a, b, torch.from_numpy(t).to(dev)))
    moved_blocks = int(((ctx.astype(np.int64) + 15) // 16).sum())
    move_bytes = 2 * moved_blocks * L * ms.block_elems * 2             # read + write
    for _ in range(3):
        binding.kv_repartition(ms, [cache], dst, cl)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = max(5, min(20, args.steps))
    ev0.record()
    for _ in range(reps):
        binding.kv_repartition(ms, [cache], dst, cl)
    ev1.record()
    torch.cuda.synchronize()
    move_ms = ev0.elapsed_time(ev1) / reps
    move_gbps = move_bytes / (move_ms * 1e-3) / 1e9

    def event_timed(fn, n):
        fn()
        torch.cuda.synchronize()
        ev0.record()
        for _ in range(n):
            fn()
        ev1.record()
        torch.cuda.synchronize()
        return ev0.elapsed_time(ev1) / n

    # What a copy reaches on this machine, timed in the same run: (a) the runtime's own device-to-device copy of about
    # the same number of bytes, contiguous; (b) this library's mover on the same blocks through IDENTITY tables
    # (block j of the pool -> block j of another pool: a contiguous copy issued by the kernel under test).
    ceil_src = cache.pool.view(-1)[: move_bytes // 4]                 # read + write = move_bytes
    ceil_dst = torch.empty_like(ceil_src)
    copy_ms = event_timed(lambda: ceil_dst.copy_(ceil_src), reps)
    del ceil_dst
    ident_lens = np.full(B, (moved_blocks // B) * 16, dtype=np.int32)   # the same blocks in total (to within B - 1), equal per sequence
    nb_i = int(ident_lens[0]) // 16
    ident_table = torch.arange(B * nb_i, dtype=torch.int32, device=dev).reshape(B, nb_i)
    id_src = binding.KVCache(cache.pool[:, : B * nb_i].contiguous(), 0, L, ident_table)
    id_dst = binding.KVCache(torch.empty_like(id_src.pool), 0, L, ident_table)
    ident_cl = torch.from_numpy(ident_lens).to(dev)
    ident_ms = event_timed(lambda: binding.kv_repartition(ms, [id_src], [id_dst], ident_cl), reps)
    ident_bytes = 2 * B * nb_i * L * ms.block_elems * 2
    del id_src, id_dst

    # ---- incremental repartition (Section 6.3: transfers run while inference continues) -----
    # (a) the snapshot pass on a second stream while decode steps run on the first: both are
    #     HBM-bound, so each slows the other; (b) a delta pass over the last 16 tokens of every
    #     sequence, the work left after 16 decode steps went by during the snapshot.
    incremental = None
    if not args.no_incremental:
        side = torch.cuda.Stream()
        reps_o = 8
        steps_o = max(1, int(round(reps_o * move_ms / ms_per_step)))      # about the same time alone
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            ev[0].record()
            for _ in range(reps_o):
                binding.kv_repartition(ms, [cache], dst, cl)
            ev[1].record()
        ev[2].record()
        for _ in range(steps_o):
            step()
        ev[3].record()
        torch.cuda.synchronize()
        move_ms_o = ev[0].elapsed_time(ev[1]) / reps_o
        step_ms_o = ev[2].elapsed_time(ev[3]) / steps_o
        delta_from = torch.clamp(cl - 16, min=0)
        for _ in range(3):
            binding.kv_repartition_range(ms, [cache], dst, delta_from, cl)
        torch.cuda.synchronize()
        ev0.record()
        for _ in range(20):
            binding.kv_repartition_range(ms, [cache], dst, delta_from, cl)
        ev1.record()
        torch.cuda.synchronize()
        delta_us = ev0.elapsed_time(ev1) / 20 * 1e3
        delta_bytes = 2 * int(np.minimum(ctx, 16).sum()) * L * kv_bytes_per_token
        incremental = {"snapshot_pass_concurrent_with_decode": {
                           "repartition_ms": move_ms_o, "repartition_GBps": move_bytes / (move_ms_o * 1e-3) / 1e9,
                           "decode_ms_per_step": step_ms_o, "decode_steps": steps_o, "repartitions": reps_o,
                           "hbm_GBps_both": (move_bytes / move_ms_o + (L * weight_bytes_layer + L * attn_bytes) / step_ms_o) / 1e6},
                       "delta_pass_last_16_tokens": {"us": delta_us, "bytes_read_plus_written": delta_bytes}}

    out = {
        # the headline configuration keeps the metric's published name; other workloads say what they are
        "metric": "stage decode tokens/s (7B shape, 4 layers, B=32); KV repartition GB/s vs HBM" if wl.name == "C2" else
                  f"stage decode tokens/s ({wl.name}: hidden {ms.hidden}, {L} layers, B={B}); KV repartition GB/s vs HBM",
        "value": tokens_per_s, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "timing": {"value_from": "median of the K steps, each timed with a HIP event pair on the launch stream",
                   "ms_per_step_wall_mean": wall_ms, "ms_per_step_min": float(np.min(step_ms)), "ms_per_step_max": float(np.max(step_ms)),
                   "first_step_of_process_ms": first_ms},
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{wl.name}: {ms.hidden}-hidden {ms.n_q_heads}/{ms.n_kv_heads}x{ms.head_dim} heads, ffn {ms.ffn}, "
                               f"{L} layers, decode batch {B}, contexts {wl.length_dist}, kv block 16, permuted block table",
                   "seed": wl.seed, "tokens_in_cache": int(ctx.sum())},
        "hbm_ideal_ms_per_step": ideal_ms, "frac_of_hbm_ideal": ideal_ms / ms_per_step,
        "kv_repartition": {"GBps": move_gbps, "ms": move_ms, "bytes_read_plus_written": move_bytes,
                           "frac_of_hbm_peak": move_gbps / HBM_PEAK_GBPS, "split": f"[0,{L}) -> [0,{half}) + [{half},{L})",
                           "copy_ceiling_GBps": move_bytes / (copy_ms * 1e-3) / 1e9,
                           "copy_ceiling": f"the runtime's device-to-device copy of {move_bytes // 2} contiguous bytes, read + write counted, same run",
                           "identity_tables_GBps": ident_bytes / (ident_ms * 1e-3) / 1e9,
                           "frac_of_copy_ceiling": move_gbps / (move_bytes / (copy_ms * 1e-3) / 1e9)},
        "roofline": {"kernel": "attn_decode_kernel", "bound": "hbm", "achieved": attn_gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": attn_gbps / HBM_PEAK_GBPS,
                     "traffic": read_traffic(os.path.join(ROOT, "profiles", "attn_decode_c2_pmc.txt"), "attn_decode_kernel"),
                     "traffic_source": "profiles/attn_decode_c2_pmc.txt (rocprofv3 --pmc runs of this command, committed; not measured in this run)",
                     "algorithmic_bytes_per_launch": attn_bytes, "avg_launch_us": attn_us},
        "incremental_repartition": incremental,
        "kernels": kernels,
        "setup_s": setup_s,
    }

    # ---- the chunked-prefill variant of the step (workload C3: 16 ragged prompts, 15,928 tokens) through the same stage:
    # the MFMA-bound side of the path, timed in the same run
    if wl.name == "C2" and not args.no_prefill:
        out["prefill"] = prefill_record(torch, synth.WORKLOADS["C3"], stage, 5, 2,
                                        weights_note="; through the decode workload's stage (same shape and depth, weights of seed 1)")

    # ---- the oracle on the host cores, on a bounded sample of the same workload ------
    if not args.no_cpu_baseline:
        import oracle
        osh = oracle.Shape(ms.hidden, ms.n_q_heads, ms.n_kv_heads, ms.head_dim, ms.ffn, 16, ms.rms_eps, ms.rope_base)
        wf = [{k: oracle.bf16_bits_to_f32(v) for k, v in lw.items()} for lw in w_bits]
        sample = list(range(B if args.cpu_sample_seqs <= 0 else min(args.cpu_sample_seqs, B)))
        nb = [(int(ctx[i]) + 16) // 16 for i in sample]
        sub_table = np.full((len(sample), max(nb)), -1, dtype=np.int32)
        blocks, at = [], 0
        for r, i in enumerate(sample):
            sub_table[r, : nb[r]] = np.arange(at, at + nb[r]); at += nb[r]
            blocks.append(table[i, : nb[r]])
        sub_pool = oracle.bf16_bits_to_f32(pool_host[:, np.concatenate(blocks)])
        xs = oracle.bf16_bits_to_f32(hidden_bits[sample]).astype(np.float64)
        # ~10 s of oracle work: the same decode step repeated (it writes the new token's K,V to the
        # same cache slots every time, so every repetition does identical work)
        cpu_reps, cpu_s = 0, 0.0
        while cpu_s < 10.0 and cpu_reps < 64:
            t0 = time.perf_counter()
            ref = oracle.stage_forward(osh, wf, sub_pool, np.arange(len(sample) + 1), ctx[sample], sub_table, xs)
            cpu_s += time.perf_counter() - t0
            cpu_reps += 1
        got = synth.bf16_bits_to_f32(y[sample].view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)
        rms = np.sqrt((ref ** 2).mean(axis=1, keepdims=True))
        out["cpu_baseline"] = {"value": len(sample) * cpu_reps / cpu_s, "unit": "tokens/s", "cores": oracle.num_threads(),
                               "kind": "oracle",
                               "sample": f"{cpu_reps} repetitions of one decode step of the same stage for {len(sample)} of the {B} "
                                         f"sequences of the batch ({int(ctx[sample].sum())} cached tokens), {cpu_s:.1f} s of oracle time",
                               "gpu_vs_oracle_rel_l2": float(np.sqrt(((got - ref) ** 2).sum(axis=1) / (ref ** 2).sum(axis=1)).max()),
                               "gpu_vs_oracle_max_elem": float((np.abs(got - ref) / np.maximum(np.abs(ref), rms)).max())}
        # the plain-loop repartition of the oracle on the same cache, same split, same tables, host memory
        osrc = [oracle.KVView(pool_host, 0, L, table)]
        odst = []
        for dv in dst:
            t_host = dv.block_table.cpu().numpy()
            odst.append(oracle.KVView(np.zeros(tuple(dv.pool.shape), dtype=np.uint16), dv.layer_begin, dv.layer_end, t_host))
        oracle.kv_repartition(osh, osrc, odst, ctx)                  # first pass touches the destination pages
        t0 = time.perf_counter()
        oracle.kv_repartition(osh, osrc, odst, ctx)
        o_s = time.perf_counter() - t0
        same = all(np.array_equal(dv.pool.cpu().numpy().view(np.uint16), od.pool) for dv, od in zip(dst, odst))
        out["kv_repartition"]["cpu_baseline"] = {"GBps": move_bytes / o_s / 1e9, "ms": o_s * 1e3, "cores": 1, "kind": "oracle",
                                                 "sample": f"the whole workload: every block of the {B} sequences, {L} layers, one pass "
                                                           "(the oracle's repartition is one plain loop on one thread)",
                                                 "gpu_equals_oracle_bit_exact": bool(same)}
    calibration_copy(torch, dev)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
