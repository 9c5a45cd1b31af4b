"""CPU oracle for the stage-forward and KV-repartition paths.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()``
and by the ``cpu_baseline`` leg of ``bench.py``.  Nothing in the GPU package
imports this module and this module imports nothing from the GPU package.

The arithmetic lives in ``flexstage_oracle.c`` (plain C loops, double
intermediates); this file only builds that file with gcc and marshals numpy
arrays into it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "flexstage_oracle.c")
_LIB = os.path.join(_HERE, "libflexstage_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP for the outer loops only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


class _Shape(C.Structure):
    _fields_ = [
        ("hidden", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
        ("head_dim", C.c_int32), ("ffn", C.c_int32), ("kv_block_size", C.c_int32),
        ("rms_eps", C.c_double), ("rope_base", C.c_double),
    ]


class _Layer(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("g_attn", "wq", "wk", "wv", "wo", "g_ffn", "w_gate", "w_up", "w_down")]


class _View(C.Structure):
    _fields_ = [
        ("base", C.c_void_p), ("num_blocks", C.c_int64),
        ("layer_begin", C.c_int32), ("layer_end", C.c_int32),
        ("block_table", C.c_void_p), ("max_blocks_per_seq", C.c_int32),
    ]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_silu.restype = C.c_double
        _lib.orc_silu.argtypes = [C.c_double]
        _lib.orc_relu.restype = C.c_double
        _lib.orc_relu.argtypes = [C.c_double]
        _lib.orc_kv_packed_elems.restype = C.c_int64
        _lib.orc_kv_packed_tokens_elems.restype = C.c_int64
    return _lib


@dataclass(frozen=True)
class Shape:
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    kv_block_size: int = 16
    rms_eps: float = 1e-5
    rope_base: float = 10000.0

    def c(self) -> _Shape:
        return _Shape(self.hidden, self.n_q_heads, self.n_kv_heads, self.head_dim, self.ffn,
                      self.kv_block_size, self.rms_eps, self.rope_base)

    @property
    def block_elems(self) -> int:
        """elements of one (layer, block) unit: K and V, all KV heads."""
        return 2 * self.n_kv_heads * self.kv_block_size * self.head_dim


def num_threads() -> int:
    return int(lib().orc_num_threads())


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a: np.ndarray) -> C.c_void_p:
    return C.c_void_p(a.ctypes.data)


# ---------------------------------------------------------------- elementary ops
def rmsnorm(x, g, eps: float) -> np.ndarray:
    x = _f64(x); g = _f32(g)
    y = np.empty_like(x)
    rows = x.reshape(-1, x.shape[-1]); out = y.reshape(-1, x.shape[-1])
    for r in range(rows.shape[0]):
        lib().orc_rmsnorm(_p(rows[r]), _p(g), C.c_int32(x.shape[-1]), C.c_double(eps), _p(out[r]))
    return y


def linear(x, W) -> np.ndarray:
    x = _f64(x); W = _f32(W)
    T, K = x.shape
    N = W.shape[0]
    assert W.shape[1] == K
    y = np.empty((T, N), dtype=np.float64)
    lib().orc_linear(_p(x), C.c_int32(T), _p(W), C.c_int32(N), C.c_int32(K), _p(y))
    return y


def rope(u, pos: int, base: float) -> np.ndarray:
    u = _f64(u).copy()
    lib().orc_rope(_p(u), C.c_int32(u.shape[-1]), C.c_int64(pos), C.c_double(base))
    return u


def silu(z: float) -> float:
    return float(lib().orc_silu(C.c_double(z)))


def softmax(s) -> np.ndarray:
    s = _f64(s).copy()
    lib().orc_softmax(_p(s), C.c_int32(s.shape[0]))
    return s


def attend_token(shape: Shape, pool: np.ndarray, layer_local: int, table_row, pos: int, q,
                 want_probs: bool = False):
    """Attention of one query token (all heads) at position ``pos`` over keys 0..pos."""
    assert pool.dtype == np.float32 and pool.flags.c_contiguous
    num_blocks = pool.shape[1]
    q = _f64(q); table_row = _i32(table_row)
    o = np.empty((shape.n_q_heads, shape.head_dim), dtype=np.float64)
    probs = np.zeros((shape.n_q_heads, pos + 1), dtype=np.float64) if want_probs else None
    sh = shape.c()
    lib().orc_attend_token(C.byref(sh), _p(pool), C.c_int64(num_blocks), C.c_int32(layer_local),
                           _p(table_row), C.c_int64(pos), _p(q), _p(o),
                           _p(probs) if want_probs else None, C.c_int64(pos + 1))
    return (o, probs) if want_probs else o


# ---------------------------------------------------------------- stage forward
LAYER_TENSORS = ("g_attn", "wq", "wk", "wv", "wo", "g_ffn", "w_gate", "w_up", "w_down")


def new_pool(shape: Shape, n_layers: int, num_blocks: int, dtype=np.float32) -> np.ndarray:
    return np.zeros((n_layers, num_blocks, 2, shape.n_kv_heads, shape.kv_block_size, shape.head_dim),
                    dtype=dtype)


def stage_forward(shape: Shape, layers: Sequence[dict], pool: np.ndarray,
                  cu_seqlens_q, ctx_lens, block_table, hidden_in,
                  probs_stride: int = 0):
    """Run the stage's layers (``layers[k]`` maps tensor name -> float32 array)
    over one ragged batch.  Appends to ``pool`` in place.  Returns hidden_out
    (float64 [T,H]) and, when ``probs_stride`` > 0, the attention probabilities
    (float64 [n_layers, T, Hq, probs_stride])."""
    assert pool.dtype == np.float32 and pool.flags.c_contiguous
    n_layers = len(layers)
    assert pool.shape[0] == n_layers
    keep = []
    arr = (_Layer * max(n_layers, 1))()
    for k, lw in enumerate(layers):
        for name in LAYER_TENSORS:
            a = _f32(lw[name]); keep.append(a)
            setattr(arr[k], name, a.ctypes.data)
    cu = _i32(cu_seqlens_q); cl = _i32(ctx_lens); bt = _i32(block_table)
    num_seqs = cl.shape[0]
    assert bt.ndim == 2 and bt.shape[0] == num_seqs and cu.shape[0] == num_seqs + 1
    x = _f64(hidden_in)
    T = int(cu[-1]) if num_seqs else 0
    assert x.shape == (T, shape.hidden)
    y = np.empty_like(x)
    probs = (np.zeros((n_layers, T, shape.n_q_heads, probs_stride), dtype=np.float64)
             if probs_stride else None)
    sh = shape.c()
    rc = lib().orc_stage_forward(
        C.byref(sh), arr, C.c_int32(n_layers), _p(pool), C.c_int64(pool.shape[1]),
        C.c_int32(num_seqs), _p(cu), _p(cl), _p(bt), C.c_int32(bt.shape[1]),
        _p(x), _p(y), _p(probs) if probs_stride else None, C.c_int64(probs_stride))
    if rc != 0:
        raise ValueError("orc_stage_forward: malformed argument")
    return (y, probs) if probs_stride else y


# ---------------------------------------------------------------- repartition
@dataclass
class KVView:
    """One stage's cache: pool array [layers][blocks][2][Hkv][bs][D] (any item
    size), the model layers it holds and the stage's block table."""
    pool: np.ndarray
    layer_begin: int
    layer_end: int
    block_table: np.ndarray

    def c(self, keep: list) -> _View:
        assert self.pool.flags.c_contiguous
        assert self.pool.shape[0] == self.layer_end - self.layer_begin
        bt = _i32(self.block_table); keep.append(bt)
        return _View(self.pool.ctypes.data, self.pool.shape[1], self.layer_begin, self.layer_end,
                     bt.ctypes.data, bt.shape[1])


def _views(vs: Sequence[KVView], keep: list):
    arr = (_View * len(vs))()
    for k, v in enumerate(vs):
        arr[k] = v.c(keep)
    return arr


def kv_repartition(shape: Shape, src: Sequence[KVView], dst: Sequence[KVView], ctx_lens) -> None:
    keep: list = []
    itemsize = src[0].pool.dtype.itemsize
    assert all(v.pool.dtype.itemsize == itemsize for v in list(src) + list(dst))
    cl = _i32(ctx_lens)
    sh = shape.c()
    rc = lib().orc_kv_repartition(C.byref(sh), C.c_int32(itemsize), _views(src, keep), C.c_int32(len(src)),
                                  _views(dst, keep), C.c_int32(len(dst)), _p(cl), C.c_int32(cl.shape[0]))
    if rc != 0:
        raise ValueError("orc_kv_repartition: layer ranges or tables malformed")


def kv_packed_elems(shape: Shape, lb: int, le: int, ctx_lens) -> int:
    cl = _i32(ctx_lens)
    sh = shape.c()
    return int(lib().orc_kv_packed_elems(C.byref(sh), C.c_int32(lb), C.c_int32(le), _p(cl), C.c_int32(cl.shape[0])))


def kv_pack(shape: Shape, src: KVView, lb: int, le: int, ctx_lens) -> np.ndarray:
    keep: list = []
    cl = _i32(ctx_lens)
    out = np.empty(kv_packed_elems(shape, lb, le, cl), dtype=src.pool.dtype)
    v = src.c(keep); sh = shape.c()
    rc = lib().orc_kv_pack(C.byref(sh), C.c_int32(src.pool.dtype.itemsize), C.byref(v), C.c_int32(lb),
                           C.c_int32(le), _p(cl), C.c_int32(cl.shape[0]), _p(out))
    if rc != 0:
        raise ValueError("orc_kv_pack: malformed argument")
    return out


def kv_unpack(shape: Shape, packed: np.ndarray, dst: KVView, lb: int, le: int, ctx_lens) -> None:
    keep: list = []
    cl = _i32(ctx_lens)
    assert packed.dtype.itemsize == dst.pool.dtype.itemsize and packed.flags.c_contiguous
    assert packed.size == kv_packed_elems(shape, lb, le, cl)
    v = dst.c(keep); sh = shape.c()
    rc = lib().orc_kv_unpack(C.byref(sh), C.c_int32(dst.pool.dtype.itemsize), _p(packed), C.byref(v),
                             C.c_int32(lb), C.c_int32(le), _p(cl), C.c_int32(cl.shape[0]))
    if rc != 0:
        raise ValueError("orc_kv_unpack: malformed argument")


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to float32."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def kv_repartition_range(shape: Shape, src: Sequence[KVView], dst: Sequence[KVView], from_lens, to_lens) -> None:
    """Incremental repartition: only tokens [from_i, to_i) of every sequence (Section 6.3, Eq. 10 with a
    per-sequence range as the validity mask)."""
    keep: list = []
    itemsize = src[0].pool.dtype.itemsize
    assert all(v.pool.dtype.itemsize == itemsize for v in list(src) + list(dst))
    fl, tl = _i32(from_lens), _i32(to_lens)
    assert fl.shape == tl.shape
    sh = shape.c()
    rc = lib().orc_kv_repartition_range(C.byref(sh), C.c_int32(itemsize), _views(src, keep), C.c_int32(len(src)),
                                        _views(dst, keep), C.c_int32(len(dst)), _p(fl), _p(tl), C.c_int32(tl.shape[0]))
    if rc != 0:
        raise ValueError("orc_kv_repartition_range: layer ranges, tables or token ranges malformed")


def kv_packed_tokens_elems(shape: Shape, lb: int, le: int, from_lens, to_lens) -> int:
    fl, tl = _i32(from_lens), _i32(to_lens)
    sh = shape.c()
    return int(lib().orc_kv_packed_tokens_elems(C.byref(sh), C.c_int32(lb), C.c_int32(le), _p(fl), _p(tl),
                                                C.c_int32(tl.shape[0])))


def kv_pack_tokens(shape: Shape, src: KVView, lb: int, le: int, from_lens, to_lens) -> np.ndarray:
    keep: list = []
    fl, tl = _i32(from_lens), _i32(to_lens)
    if np.any(fl < 0) or np.any(fl > tl):
        raise ValueError("orc_kv_pack_tokens: malformed token range")
    out = np.empty(kv_packed_tokens_elems(shape, lb, le, fl, tl), dtype=src.pool.dtype)
    v = src.c(keep); sh = shape.c()
    rc = lib().orc_kv_pack_tokens(C.byref(sh), C.c_int32(src.pool.dtype.itemsize), C.byref(v), C.c_int32(lb),
                                  C.c_int32(le), _p(fl), _p(tl), C.c_int32(tl.shape[0]), _p(out))
    if rc != 0:
        raise ValueError("orc_kv_pack_tokens: malformed argument")
    return out


def kv_unpack_tokens(shape: Shape, packed: np.ndarray, dst: KVView, lb: int, le: int, from_lens, to_lens) -> None:
    keep: list = []
    fl, tl = _i32(from_lens), _i32(to_lens)
    assert packed.dtype.itemsize == dst.pool.dtype.itemsize and packed.flags.c_contiguous
    if np.any(fl < 0) or np.any(fl > tl):
        raise ValueError("orc_kv_unpack_tokens: malformed token range")
    assert packed.size == kv_packed_tokens_elems(shape, lb, le, fl, tl)
    v = dst.c(keep); sh = shape.c()
    rc = lib().orc_kv_unpack_tokens(C.byref(sh), C.c_int32(dst.pool.dtype.itemsize), _p(packed), C.byref(v),
                                    C.c_int32(lb), C.c_int32(le), _p(fl), _p(tl), C.c_int32(tl.shape[0]))
    if rc != 0:
        raise ValueError("orc_kv_unpack_tokens: malformed argument")


# ---------------------------------------------------------------- OPT-style layer
OPT_LAYER_TENSORS = ("ln1_g", "ln1_b", "wq", "bq", "wk", "bk", "wv", "bv", "wo", "bo",
                     "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")


class _OptLayer(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in OPT_LAYER_TENSORS]


def layernorm(x, g, b, eps: float) -> np.ndarray:
    x = _f64(x); g = _f32(g); b = _f32(b)
    y = np.empty_like(x)
    rows = x.reshape(-1, x.shape[-1]); out = y.reshape(-1, x.shape[-1])
    for r in range(rows.shape[0]):
        lib().orc_layernorm(_p(rows[r]), _p(g), _p(b), C.c_int32(x.shape[-1]), C.c_double(eps), _p(out[r]))
    return y


def linear_bias(x, W, bias) -> np.ndarray:
    x = _f64(x); W = _f32(W); bias = _f32(bias)
    T, K = x.shape
    N = W.shape[0]
    assert W.shape[1] == K and bias.shape == (N,)
    y = np.empty((T, N), dtype=np.float64)
    lib().orc_linear_bias(_p(x), C.c_int32(T), _p(W), _p(bias), C.c_int32(N), C.c_int32(K), _p(y))
    return y


def relu(z: float) -> float:
    return float(lib().orc_relu(C.c_double(z)))


def stage_forward_opt(shape: Shape, layers: Sequence[dict], pool: np.ndarray,
                      cu_seqlens_q, ctx_lens, block_table, hidden_in, probs_stride: int = 0):
    """stage_forward for OPT-style layers (``layers[k]`` maps the OPT_LAYER_TENSORS names to
    float32 arrays); ``shape.rms_eps`` is the LayerNorm epsilon."""
    assert pool.dtype == np.float32 and pool.flags.c_contiguous
    n_layers = len(layers)
    assert pool.shape[0] == n_layers
    keep = []
    arr = (_OptLayer * max(n_layers, 1))()
    for k, lw in enumerate(layers):
        for name in OPT_LAYER_TENSORS:
            a = _f32(lw[name]); keep.append(a)
            setattr(arr[k], name, a.ctypes.data)
    cu = _i32(cu_seqlens_q); cl = _i32(ctx_lens); bt = _i32(block_table)
    num_seqs = cl.shape[0]
    assert bt.ndim == 2 and bt.shape[0] == num_seqs and cu.shape[0] == num_seqs + 1
    x = _f64(hidden_in)
    T = int(cu[-1]) if num_seqs else 0
    assert x.shape == (T, shape.hidden)
    y = np.empty_like(x)
    probs = (np.zeros((n_layers, T, shape.n_q_heads, probs_stride), dtype=np.float64) if probs_stride else None)
    sh = shape.c()
    rc = lib().orc_stage_forward_opt(
        C.byref(sh), arr, C.c_int32(n_layers), _p(pool), C.c_int64(pool.shape[1]),
        C.c_int32(num_seqs), _p(cu), _p(cl), _p(bt), C.c_int32(bt.shape[1]),
        _p(x), _p(y), _p(probs) if probs_stride else None, C.c_int64(probs_stride))
    if rc != 0:
        raise ValueError("orc_stage_forward_opt: malformed argument")
    return (y, probs) if probs_stride else y
