"""Seeded synthetic inputs for the stage-forward / KV-repartition workloads.

This module only *draws* inputs (weights, lengths, block tables, hidden states,
cache contents) and encodes them as bf16 bit patterns.  It contains none of the
method's arithmetic and is the one module both the GPU tests and the CPU-side
checks read their inputs from.  Everything is derived from
``numpy.random.Generator(PCG64(...))`` seeded by (config seed, stream tag,
index), so any single layer or sequence can be regenerated on its own.

The paper measures on production request traces that are not distributed with
it; the five workloads below (shapes of public Llama-family models, stated
length distributions) stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Tuple

import numpy as np

LAYER_TENSORS = ("g_attn", "wq", "wk", "wv", "wo", "g_ffn", "w_gate", "w_up", "w_down")

# stream tags for the per-purpose generators
_TAG_WEIGHT, _TAG_LENS, _TAG_PERM, _TAG_HIDDEN, _TAG_CACHE, _TAG_OPT_WEIGHT = 1, 2, 3, 4, 5, 6


@dataclass(frozen=True)
class ModelShape:
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    kv_block_size: int = 16
    arch: int = 0          # 0: Llama-style layer (RMSNorm, rotary, SwiGLU); 1: OPT-style (LayerNorm, biases, ReLU)

    @property
    def qkv_out(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    @property
    def block_elems(self) -> int:
        """bf16 elements of one (layer, block) unit: K and V, all KV heads."""
        return 2 * self.n_kv_heads * self.kv_block_size * self.head_dim

    @property
    def params_per_layer(self) -> int:
        H, D, F = self.hidden, self.head_dim, self.ffn
        if self.arch == 1:
            return self.qkv_out * H + H * self.n_q_heads * D + 2 * F * H + self.qkv_out + 2 * H + F + 4 * H
        return (self.qkv_out * H + H * self.n_q_heads * D + 3 * F * H + 2 * H)


@dataclass(frozen=True)
class Workload:
    name: str
    seed: int
    shape: ModelShape
    n_layers: int
    num_seqs: int
    kind: str            # "decode" or "prefill"
    length_dist: Tuple   # see draw_lengths


TINY = ModelShape(hidden=256, n_q_heads=4, n_kv_heads=4, head_dim=64, ffn=688)
TINY_OPT = ModelShape(hidden=256, n_q_heads=4, n_kv_heads=4, head_dim=64, ffn=1024, arch=1)
OPT_66B = ModelShape(hidden=9216, n_q_heads=72, n_kv_heads=72, head_dim=128, ffn=36864, arch=1)
LLAMA2_7B = ModelShape(hidden=4096, n_q_heads=32, n_kv_heads=32, head_dim=128, ffn=11008)
LLAMA2_13B = ModelShape(hidden=5120, n_q_heads=40, n_kv_heads=40, head_dim=128, ffn=13824)
LLAMA3_70B = ModelShape(hidden=8192, n_q_heads=64, n_kv_heads=8, head_dim=128, ffn=28672)

WORKLOADS: Dict[str, Workload] = {
    "C1": Workload("C1", 0, TINY, 2, 4, "decode", ("uniform", 32, 128)),
    "C2": Workload("C2", 1, LLAMA2_7B, 4, 32, "decode", ("uniform", 512, 4096)),
    "C3": Workload("C3", 2, LLAMA2_7B, 4, 16, "prefill", ("loguniform", 256, 2048)),
    "C4": Workload("C4", 3, LLAMA2_13B, 8, 64, "decode", ("lognormal", 1024, 0.8, 64, 8192)),
    "C5": Workload("C5", 4, LLAMA3_70B, 4, 128, "decode", ("uniform", 1024, 8192)),
}


def _rng(seed: int, tag: int, *index: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([seed, tag, *index]))


# ---------------------------------------------------------------- bf16 encoding
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round-to-nearest-even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


_CHUNK = 1 << 20


def _normal_bf16(g: np.random.Generator, shape, scale: float = 1.0, offset: float = 0.0) -> np.ndarray:
    """bf16 bit patterns of ``offset + scale * N(0,1)`` drawn from ``g`` in float32 and rounded to
    nearest even: the values of ``f32_to_bf16_bits(g.standard_normal(shape, float32) * scale + offset)``,
    produced a chunk at a time in reused buffers (large temporaries cost more than the draw itself)."""
    n = int(np.prod(shape, dtype=np.int64))
    out = np.empty(n, dtype=np.uint16)
    buf = np.empty(min(n, _CHUNK), dtype=np.float32)
    tmp = np.empty(min(n, _CHUNK), dtype=np.uint32)
    for at in range(0, n, _CHUNK):
        m = min(_CHUNK, n - at)
        a, t = buf[:m], tmp[:m]
        g.standard_normal(out=a, dtype=np.float32)
        if scale != 1.0:
            a *= np.float32(scale)
        if offset != 0.0:
            a += np.float32(offset)
        u = a.view(np.uint32)
        np.right_shift(u, np.uint32(16), out=t)
        t &= np.uint32(1)
        t += np.uint32(0x7FFF)
        u += t
        u >>= np.uint32(16)
        out[at:at + m] = u
    return out.reshape(shape)


# ---------------------------------------------------------------- draws
def layer_weights(shape: ModelShape, seed: int, layer: int) -> Dict[str, np.ndarray]:
    """bf16 bit patterns of one decoder layer's tensors.  Projection matrices
    ~ N(0, 0.02), stored [out_features][in_features]; norm gains 1 + N(0, 0.02)."""
    g = _rng(seed, _TAG_WEIGHT, layer)
    H, D, F = shape.hidden, shape.head_dim, shape.ffn
    dims = {
        "g_attn": (H,), "wq": (shape.n_q_heads * D, H), "wk": (shape.n_kv_heads * D, H),
        "wv": (shape.n_kv_heads * D, H), "wo": (H, shape.n_q_heads * D), "g_ffn": (H,),
        "w_gate": (F, H), "w_up": (F, H), "w_down": (H, F),
    }
    out = {}
    for name in LAYER_TENSORS:
        out[name] = _normal_bf16(g, dims[name], 0.02, 1.0 if name.startswith("g_") else 0.0)
    return out


OPT_LAYER_TENSORS = ("ln1_g", "ln1_b", "wq", "bq", "wk", "bk", "wv", "bv", "wo", "bo",
                     "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")


def opt_layer_weights(shape: ModelShape, seed: int, layer: int) -> Dict[str, np.ndarray]:
    """bf16 bit patterns of one OPT-style layer: matrices and biases ~ N(0, 0.02), LayerNorm gains
    1 + N(0, 0.02)."""
    g = _rng(seed, _TAG_OPT_WEIGHT, layer)
    H, D, F = shape.hidden, shape.head_dim, shape.ffn
    Nq, Nkv = shape.n_q_heads * D, shape.n_kv_heads * D
    dims = {
        "ln1_g": (H,), "ln1_b": (H,), "wq": (Nq, H), "bq": (Nq,), "wk": (Nkv, H), "bk": (Nkv,), "wv": (Nkv, H), "bv": (Nkv,),
        "wo": (H, Nq), "bo": (H,), "ln2_g": (H,), "ln2_b": (H,), "w_fc1": (F, H), "b_fc1": (F,), "w_fc2": (H, F), "b_fc2": (H,),
    }
    out = {}
    for name in OPT_LAYER_TENSORS:
        out[name] = _normal_bf16(g, dims[name], 0.02, 1.0 if name.endswith("_g") else 0.0)
    return out


def draw_lengths(dist: Tuple, n: int, seed: int) -> np.ndarray:
    g = _rng(seed, _TAG_LENS)
    kind = dist[0]
    if kind == "uniform":          # integers uniform in [lo, hi]
        return g.integers(dist[1], dist[2] + 1, size=n).astype(np.int32)
    if kind == "loguniform":       # round(exp(U(ln lo, ln hi)))
        return np.rint(np.exp(g.uniform(np.log(dist[1]), np.log(dist[2]), size=n))).astype(np.int32)
    if kind == "lognormal":        # clip(round(exp(N(ln median, sigma^2))), lo, hi)
        _, median, sigma, lo, hi = dist
        return np.clip(np.rint(np.exp(g.normal(np.log(median), sigma, size=n))), lo, hi).astype(np.int32)
    raise ValueError(kind)


def blocks_for(tokens: np.ndarray, block_size: int) -> np.ndarray:
    return (np.asarray(tokens, dtype=np.int64) + block_size - 1) // block_size


def block_table(tokens_after: np.ndarray, block_size: int, seed: int, salt: int = 0,
                spare_blocks: int = 0) -> Tuple[np.ndarray, int]:
    """A block table with room for ``tokens_after[i]`` tokens per sequence, whose
    physical ids are a random permutation of the pool.  Unused entries are -1.
    Returns (table int32 [num_seqs, max_blocks], num_blocks in the pool)."""
    need = blocks_for(tokens_after, block_size)
    total = int(need.sum()) + int(spare_blocks)
    perm = _rng(seed, _TAG_PERM, salt).permutation(total).astype(np.int32)
    max_blocks = int(need.max()) if need.size else 0
    table = np.full((len(need), max(max_blocks, 1)), -1, dtype=np.int32)
    at = 0
    for i, nb in enumerate(need):
        table[i, :nb] = perm[at:at + nb]
        at += int(nb)
    return table, max(total, 1)


def hidden_states(num_tokens: int, hidden: int, seed: int, salt: int = 0) -> np.ndarray:
    """bf16 bit patterns of N(0,1) hidden rows, [num_tokens, hidden]."""
    return _normal_bf16(_rng(seed, _TAG_HIDDEN, salt), (num_tokens, hidden))


def cache_rows(shape: ModelShape, seed: int, seq: int, layer: int, n_tokens: int) -> np.ndarray:
    """Synthetic cache contents of one (sequence, layer): bf16 bit patterns of
    N(0,1) values, [n_tokens][2: K,V][kv_head][head_dim]."""
    return _normal_bf16(_rng(seed, _TAG_CACHE, seq, layer), (n_tokens, 2, shape.n_kv_heads, shape.head_dim))


def fill_pool_rows(pool: np.ndarray, layer_local: int, table_row: np.ndarray, rows: np.ndarray,
                   block_size: int) -> None:
    """Write ``rows`` ([n_tokens][2][Hkv][D], any dtype matching ``pool``) of one
    sequence into ``pool`` [layers][blocks][2][Hkv][bs][D] through its table row.
    Pure placement (no arithmetic)."""
    n = rows.shape[0]
    for j in range((n + block_size - 1) // block_size):
        lo, hi = j * block_size, min(n, (j + 1) * block_size)
        # rows[lo:hi] is [slot][kv][head][D] -> pool block is [kv][head][slot][D]
        pool[layer_local, table_row[j], :, :, : hi - lo, :] = np.transpose(rows[lo:hi], (1, 2, 0, 3))


def cu_seqlens(q_lens: np.ndarray) -> np.ndarray:
    out = np.zeros(len(q_lens) + 1, dtype=np.int32)
    np.cumsum(q_lens, out=out[1:])
    return out
