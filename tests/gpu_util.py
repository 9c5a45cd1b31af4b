"""Helpers shared by the GPU parity tests: build a synthetic workload once on
the host (bf16 bit patterns from ``synth``), hand the same bits to the oracle
(widened to float32) and to the GPU library (uploaded as bf16)."""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

import oracle
from paper_2510_11938_amd import binding, synth


def oracle_shape(ms: synth.ModelShape) -> oracle.Shape:
    return oracle.Shape(ms.hidden, ms.n_q_heads, ms.n_kv_heads, ms.head_dim, ms.ffn,
                        ms.kv_block_size, ms.rms_eps, ms.rope_base)


def dev_bf16(bits: np.ndarray) -> torch.Tensor:
    """uint16 bit patterns -> CUDA bfloat16 tensor of the same shape."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def host_bits(t: torch.Tensor) -> np.ndarray:
    """CUDA bf16/int16 tensor -> uint16 numpy array."""
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def host_f64(t: torch.Tensor) -> np.ndarray:
    return synth.bf16_bits_to_f32(host_bits(t)).astype(np.float64)


def dev_i32(a) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def rel_err(gpu: np.ndarray, ref: np.ndarray) -> float:
    """max_e |g - o| / max(|o|, rms(o_row)): the stage-output error measure."""
    rms = np.sqrt((ref ** 2).mean(axis=-1, keepdims=True))
    return float((np.abs(gpu - ref) / np.maximum(np.abs(ref), rms)).max())


@dataclass
class Weights:
    bits: List[Dict[str, np.ndarray]]         # per layer: name -> uint16 bf16 patterns
    f32: List[Dict[str, np.ndarray]]          # the same values as float32 (oracle input)
    dev: List[Dict[str, torch.Tensor]]        # CUDA bf16 tensors


def make_weights(ms: synth.ModelShape, seed: int, n_layers: int, want_f32: bool = True, want_dev: bool = True) -> Weights:
    gen = synth.opt_layer_weights if ms.arch == 1 else synth.layer_weights
    with ThreadPoolExecutor(max_workers=8) as ex:             # layers have generators of their own: drawn side by side
        bits = list(ex.map(lambda l: gen(ms, seed, l), range(n_layers)))
    f32 = [{k: synth.bf16_bits_to_f32(v) for k, v in lw.items()} for lw in bits] if want_f32 else []
    dev = [{k: dev_bf16(v) for k, v in lw.items()} for lw in bits] if want_dev else []
    return Weights(bits, f32, dev)


def filled_pool_bits(ms: synth.ModelShape, seed: int, n_layers: int, ctx_lens: np.ndarray, table: np.ndarray,
                     num_blocks: int, layer0: int = 0, seqs: Optional[Sequence[int]] = None,
                     threads: int = 8) -> np.ndarray:
    """Host pool [layers][blocks][2][Hkv][16][D] of bf16 bits, zero except for the
    synthetic cache rows of the given sequences (default: all)."""
    pool = np.zeros((n_layers, num_blocks, 2, ms.n_kv_heads, ms.kv_block_size, ms.head_dim), dtype=np.uint16)
    todo = [(i, l) for i in (range(len(ctx_lens)) if seqs is None else seqs) for l in range(n_layers)]

    def one(job):
        i, l = job
        rows = synth.cache_rows(ms, seed, i, layer0 + l, int(ctx_lens[i]))
        synth.fill_pool_rows(pool, l, table[i], rows, ms.kv_block_size)

    with ThreadPoolExecutor(max_workers=threads) as ex:
        list(ex.map(one, todo))
    return pool


def oracle_forward(ms: synth.ModelShape):
    """The oracle's stage function for the model's layer kind."""
    return oracle.stage_forward_opt if ms.arch == 1 else oracle.stage_forward


def pool_f32(bits: np.ndarray) -> np.ndarray:
    return synth.bf16_bits_to_f32(bits)


def make_stage(ms: synth.ModelShape, w: Weights, lb: int, le: int) -> binding.Stage:
    return binding.Stage(ms, lb, le, w.dev[lb:le])
