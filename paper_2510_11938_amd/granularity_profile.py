"""Stage time against stage depth, and the granularity the controller would pick.

The method chooses between pipeline granularities from their throughput T_k and latency
L_k (Section 6.1, Eq. 4); the paper tabulates per-stage compute and communication time for
several stage counts (Table 2).  This script measures the compute side on the GPU it runs
on -- one decode step of a stage of 1, 2, 4, 8 ... layers through fxp_stage_forward -- and
models the hand-off between stages (one [batch, hidden] bf16 transfer per step over a link of
given bandwidth and latency).  With one GPU per stage and the pipeline full,
    T_k = batch / (t_stage + t_handoff)          tokens/s
    L_k = n_stages * (t_stage + t_handoff)       seconds per token through the pipeline
and fxp_ctl_select_granularity scores the candidates for a range of traffic CVs.

    python -m paper_2510_11938_amd.granularity_profile --layers-total 32 --depths 1,2,4,8

Inputs are synthetic (random weights and cache contents; only the sizes matter for time).
"""
from __future__ import annotations

import argparse
import json
import sys

import numpy as np
import torch

from . import binding, synth


def measure_stage_ms(ms: synth.ModelShape, depth: int, batch: int, ctx: np.ndarray, steps: int) -> float:
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev); g.manual_seed(depth)

    def rnd(*shape, scale=0.02):
        return (torch.randn(*shape, device=dev, generator=g) * scale).to(torch.bfloat16)

    H, D, F = ms.hidden, ms.head_dim, ms.ffn
    Nq, Nkv = ms.n_q_heads * D, ms.n_kv_heads * D
    if ms.arch == binding.ARCH_OPT:
        layers = [dict(ln1_g=1 + rnd(H), ln1_b=rnd(H), wq=rnd(Nq, H), bq=rnd(Nq), wk=rnd(Nkv, H), bk=rnd(Nkv), wv=rnd(Nkv, H),
                       bv=rnd(Nkv), wo=rnd(H, Nq), bo=rnd(H), ln2_g=1 + rnd(H), ln2_b=rnd(H), w_fc1=rnd(F, H), b_fc1=rnd(F),
                       w_fc2=rnd(H, F), b_fc2=rnd(H)) for _ in range(depth)]
    else:
        layers = [dict(g_attn=1 + rnd(H), wq=rnd(Nq, H), wk=rnd(Nkv, H), wv=rnd(Nkv, H), wo=rnd(H, Nq), g_ffn=1 + rnd(H),
                       w_gate=rnd(F, H), w_up=rnd(F, H), w_down=rnd(H, F)) for _ in range(depth)]
    stage = binding.Stage(ms, 0, depth, layers)
    torch.cuda.synchronize()
    del layers
    table, nblk = synth.block_table(ctx + 1, 16, seed=depth)
    pool = torch.empty((depth, nblk, 2, ms.n_kv_heads, 16, D), dtype=torch.bfloat16, device=dev).normal_(generator=g)
    cache = binding.KVCache(pool, 0, depth, torch.from_numpy(table).to(dev))
    x = rnd(batch, H, scale=1.0)
    y = torch.empty_like(x)
    cu = torch.arange(batch + 1, dtype=torch.int32, device=dev)
    cl = torch.from_numpy(ctx).to(dev)
    for _ in range(3):
        stage.forward(cache, cu, cl, x, 1, hidden_out=y)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        stage.forward(cache, cu, cl, x, 1, hidden_out=y)
    e1.record()
    torch.cuda.synchronize()
    stage.close()
    return e0.elapsed_time(e1) / steps


def layer_tensor_shapes(ms: synth.ModelShape) -> dict:
    H, D, F = ms.hidden, ms.head_dim, ms.ffn
    Nq, Nkv = ms.n_q_heads * D, ms.n_kv_heads * D
    if ms.arch == binding.ARCH_OPT:
        return dict(ln1_g=(H,), ln1_b=(H,), wq=(Nq, H), bq=(Nq,), wk=(Nkv, H), bk=(Nkv,), wv=(Nkv, H), bv=(Nkv,), wo=(H, Nq), bo=(H,),
                    ln2_g=(H,), ln2_b=(H,), w_fc1=(F, H), b_fc1=(F,), w_fc2=(H, F), b_fc2=(H,))
    return dict(g_attn=(H,), wq=(Nq, H), wk=(Nkv, H), wv=(Nkv, H), wo=(H, Nq), g_ffn=(H,), w_gate=(F, H), w_up=(F, H), w_down=(H, F))


def load_stage(ms: synth.ModelShape, host_layers, layer_begin: int = 0):
    """A stage's parameters from pinned host memory (``host_layers``: one dict of pinned bf16 CPU tensors per
    layer, named as binding.Stage expects) to the GPU, then fxp_stage_create's re-tiling into the stage's
    arena.  Returns (stage, host -> GPU ms, re-tile ms)."""
    dev = torch.device("cuda:0")
    for lw in host_layers:
        assert all(t.is_pinned() for t in lw.values())
    e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    e[0].record()
    layers = [{k: t.to(dev, non_blocking=True) for k, t in lw.items()} for lw in host_layers]
    e[1].record()
    stage = binding.Stage(ms, layer_begin, layer_begin + len(host_layers), layers)
    e[2].record()
    torch.cuda.synchronize()
    return stage, e[0].elapsed_time(e[1]), e[1].elapsed_time(e[2])


def measure_load_ms(ms: synth.ModelShape, depth: int) -> dict:
    """The load column of Table 2 as far as one GPU can show it: a stage's parameters go from pinned
    host memory to the GPU (one layer's worth of pinned buffers, copied once per layer: the contents do
    not matter for the time) and fxp_stage_create re-tiles them into the stage's arena."""
    shapes = layer_tensor_shapes(ms)
    host = {k: torch.zeros(shp, dtype=torch.bfloat16).pin_memory() for k, shp in shapes.items()}
    layer_bytes = sum(t.numel() * 2 for t in host.values())
    torch.cuda.synchronize()
    stage, h2d_ms, retile_ms = load_stage(ms, [host] * depth)
    stage.close()
    return {"bytes": layer_bytes * depth, "h2d_ms": h2d_ms, "retile_ms": retile_ms}


def max_batch(ms: synth.ModelShape, depth: int, ctx_len: int, hbm_bytes: float) -> int:
    """Sequences of ctx_len cached tokens whose KV blocks fit next to the stage's weights (raw + re-tiled are not
    both kept: the arena alone stays) in hbm_bytes."""
    weights = ms.params_per_layer * 2 * depth
    per_seq = -(-(ctx_len + 1) // 16) * ms.block_elems * 2 * depth
    return int(max(0.0, hbm_bytes - weights) // per_seq)


def stage_candidate(layers_total: int, depth: int, batch: int, compute_ms: float, handoff_ms: float) -> binding.Granularity:
    """The candidate g_k = (eta_k stages, batch b_k) of Eq. 4 from a measured stage time: with one GPU per stage and
    the pipeline full, T_k = batch / (t_stage + t_handoff) tokens/s and L_k = eta_k (t_stage + t_handoff) ms."""
    n_stages = layers_total // depth
    return binding.Granularity(n_stages, batch, batch / ((compute_ms + handoff_ms) * 1e-3), n_stages * (compute_ms + handoff_ms), 0.0)


def spread_cv_opt(cands, cvs) -> None:
    """nu_k: finer granularities suit burstier traffic; the candidates are spread over the CVs scored."""
    order = np.argsort([c.n_stages for c in cands])
    for rank, k in enumerate(order):
        cands[k].cv_opt = cvs[min(rank * len(cvs) // len(cands), len(cvs) - 1)]


def select_for_cvs(cands, cvs, alpha: float, sigma: float):
    """fxp_ctl_select_granularity (Eq. 4) at each traffic CV."""
    picks = []
    for cv in cvs:
        best, scores = binding.ctl_select_granularity(cands, cv, alpha, sigma)
        picks.append({"cv": cv, "selected_n_stages": cands[best].n_stages, "scores": scores})
    return picks


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--model", default="7b", choices=["7b", "opt66b"],
                    help="7b: Llama-style 7B shape (32 layers); opt66b: OPT-66B shape (64 layers), the model of the paper's Table 2")
    ap.add_argument("--layers-total", type=int, default=0, help="layers of the whole model (default: the model's own)")
    ap.add_argument("--depths", default="1,2,4,8", help="layers per stage to measure")
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--ctx", default="512,4096", help="uniform context length range")
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--link-gbps", type=float, default=153.0, help="stage-to-stage link, GB/s (one xGMI link)")
    ap.add_argument("--link-latency-us", type=float, default=10.0)
    ap.add_argument("--alpha", type=float, default=0.5)
    ap.add_argument("--sigma", type=float, default=1.0)
    ap.add_argument("--cvs", default="0.25,1,2,4", help="traffic CVs to score")
    ap.add_argument("--load", action="store_true", help="also time host-pinned -> GPU parameter load and re-tiling per stage")
    ap.add_argument("--hbm-gb", type=float, default=288.0, help="device memory for the max-batch column")
    args = ap.parse_args(argv)
    ms = synth.OPT_66B if args.model == "opt66b" else synth.LLAMA2_7B
    if args.layers_total <= 0:
        args.layers_total = 64 if args.model == "opt66b" else 32
    lo, hi = (int(v) for v in args.ctx.split(","))
    ctx = synth.draw_lengths(("uniform", lo, hi), args.batch, seed=1)
    handoff_ms = (args.batch * ms.hidden * 2 / (args.link_gbps * 1e9) + args.link_latency_us * 1e-6) * 1e3
    rows, cands = [], []
    depths = [int(v) for v in args.depths.split(",")]
    for depth in depths:
        n_stages = args.layers_total // depth
        t = measure_stage_ms(ms, depth, args.batch, ctx, args.steps)
        cand = stage_candidate(args.layers_total, depth, args.batch, t, handoff_ms)
        thr, lat = cand.throughput, cand.latency
        rows.append({"layers_per_stage": depth, "n_stages": n_stages, "compute_ms": t, "handoff_ms": handoff_ms,
                     "throughput_tokens_s": thr, "latency_ms": lat, "max_batch_at_ctx_hi": max_batch(ms, depth, hi, args.hbm_gb * 1e9)})
        print(f"depth {depth:2d}: {n_stages:2d} stages, compute {t:7.3f} ms, hand-off {handoff_ms:6.3f} ms, "
              f"T = {thr:9.0f} tokens/s, L = {lat:7.2f} ms", file=sys.stderr, flush=True)
        if args.load:
            rows[-1]["load"] = measure_load_ms(ms, depth)
            print(f"          load {rows[-1]['load']['bytes'] / 1e9:6.2f} GB: host -> GPU {rows[-1]['load']['h2d_ms']:8.1f} ms, "
                  f"re-tile {rows[-1]['load']['retile_ms']:7.1f} ms; max batch at ctx {hi}: {rows[-1]['max_batch_at_ctx_hi']}",
                  file=sys.stderr, flush=True)
        cands.append(cand)
    cvs = [float(v) for v in args.cvs.split(",")]
    spread_cv_opt(cands, cvs)
    picks = select_for_cvs(cands, cvs, args.alpha, args.sigma)
    print(json.dumps({"model": args.model, "batch": args.batch, "ctx_range": [lo, hi], "stages": rows,
                      "cv_opt": [c.cv_opt for c in cands], "alpha": args.alpha, "sigma": args.sigma, "picks": picks}))
    return 0


if __name__ == "__main__":
    sys.exit(main())
