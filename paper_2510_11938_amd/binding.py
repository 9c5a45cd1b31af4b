"""Thin ctypes binding over the C ABI declared in ``include/flexstage.h``.

Argument marshalling only: torch tensors supply device memory and the current
HIP stream; every step of the path runs inside ``libflexstage.so``.  The
library must have been built (``python -m paper_2510_11938_amd.build``); a
missing library is an error, there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# the library this binding opens (a kernel experiment may assign another build's path here before the first call)
LIB_PATH = os.path.join(_HERE, "libflexstage.so")

FXP_OK, FXP_EINVAL, FXP_ENOSPC, FXP_EHIP = 0, -1, -2, -3

EXPORTS = (
    "fxp_stage_weight_arena_bytes", "fxp_stage_create", "fxp_stage_destroy",
    "fxp_stage_workspace_bytes", "fxp_stage_forward", "fxp_stage_forward_static", "fxp_stage_forward_debug",
    "fxp_stage_split", "fxp_stage_merge", "fxp_stage_layers",
    "fxp_kv_repartition", "fxp_kv_packed_bytes", "fxp_kv_pack", "fxp_kv_unpack",
    "fxp_kv_repartition_range", "fxp_kv_packed_tokens_bytes", "fxp_kv_pack_tokens", "fxp_kv_unpack_tokens",
    "fxp_ctl_cv", "fxp_ctl_select_granularity", "fxp_ctl_parallel_instances", "fxp_ctl_multiplexing_penalty",
    "fxp_ctl_scaling_granularity", "fxp_ctl_slo_satisfied",
    "fxp_profile_enable", "fxp_profile_num_classes", "fxp_profile_class_name", "fxp_profile_read", "fxp_profile_read_launch",
    "fxp_last_error", "fxp_version",
)


class Granularity(C.Structure):
    _fields_ = [("n_stages", C.c_int32), ("batch", C.c_int32), ("throughput", C.c_double), ("latency", C.c_double),
                ("cv_opt", C.c_double)]


class FxpError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"flexstage error {code}: {message}")
        self.code = code


class StageDesc(C.Structure):
    _fields_ = [
        ("layer_begin", C.c_int32), ("layer_end", C.c_int32), ("hidden", C.c_int32),
        ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("ffn", C.c_int32), ("rms_eps", C.c_float), ("rope_base", C.c_float),
        ("kv_block_size", C.c_int32), ("arch", C.c_int32),
    ]


ARCH_LLAMA, ARCH_OPT = 0, 1
LAYER_TENSORS = ("g_attn", "wq", "wk", "wv", "wo", "g_ffn", "w_gate", "w_up", "w_down")
BIAS_TENSORS = ("b_attn_norm", "b_ffn_norm", "bq", "bk", "bv", "bo", "b_up", "b_down")
# an OPT-style layer's tensors by their usual names -> fields of fxp_layer_weights
OPT_TENSOR_FIELDS = {"ln1_g": "g_attn", "ln1_b": "b_attn_norm", "wq": "wq", "bq": "bq", "wk": "wk", "bk": "bk", "wv": "wv", "bv": "bv",
                     "wo": "wo", "bo": "bo", "ln2_g": "g_ffn", "ln2_b": "b_ffn_norm", "w_fc1": "w_up", "b_fc1": "b_up",
                     "w_fc2": "w_down", "b_fc2": "b_down"}


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in LAYER_TENSORS + BIAS_TENSORS]


class KvPool(C.Structure):
    _fields_ = [("base", C.c_void_p), ("num_blocks", C.c_int64),
                ("layer_begin", C.c_int32), ("layer_end", C.c_int32)]


class Batch(C.Structure):
    _fields_ = [
        ("num_seqs", C.c_int32), ("num_tokens", C.c_int32), ("max_q_len", C.c_int32),
        ("max_blocks_per_seq", C.c_int32),
        ("cu_seqlens_q", C.c_void_p), ("ctx_lens", C.c_void_p), ("block_table", C.c_void_p),
        ("min_q_len", C.c_int32),
    ]


class KvView(C.Structure):
    _fields_ = [("pool", C.POINTER(KvPool)), ("block_table", C.c_void_p),
                ("max_blocks_per_seq", C.c_int32)]


_lib = None


def lib() -> C.CDLL:
    """Open libflexstage.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2510_11938_amd.build` "
                "(there is no CPU fallback)")
        l = C.CDLL(LIB_PATH)
        l.fxp_last_error.restype = C.c_char_p
        l.fxp_version.restype = C.c_char_p
        l.fxp_stage_weight_arena_bytes.restype = C.c_size_t
        l.fxp_stage_weight_arena_bytes.argtypes = [C.POINTER(StageDesc)]
        l.fxp_stage_create.argtypes = [C.POINTER(StageDesc), C.POINTER(LayerWeights), C.c_void_p, C.c_size_t,
                                       C.c_void_p, C.POINTER(C.c_void_p)]
        l.fxp_stage_destroy.argtypes = [C.c_void_p]
        l.fxp_stage_split.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p)]
        l.fxp_stage_merge.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p)]
        l.fxp_stage_layers.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        l.fxp_stage_workspace_bytes.restype = C.c_size_t
        l.fxp_stage_workspace_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32]
        l.fxp_stage_forward.argtypes = [C.c_void_p, C.POINTER(KvPool), C.POINTER(Batch), C.c_void_p, C.c_void_p,
                                        C.c_void_p, C.c_size_t, C.c_void_p]
        l.fxp_stage_forward_static.argtypes = [C.c_void_p, C.POINTER(KvPool), C.POINTER(Batch), C.c_void_p, C.c_void_p, C.c_void_p]
        l.fxp_stage_forward_debug.argtypes = [C.c_void_p, C.POINTER(KvPool), C.POINTER(Batch), C.c_void_p, C.c_void_p,
                                              C.c_void_p, C.c_size_t, C.c_void_p, C.c_int64, C.c_void_p]
        l.fxp_kv_repartition.argtypes = [C.POINTER(StageDesc), C.POINTER(KvView), C.c_int32, C.POINTER(KvView),
                                         C.c_int32, C.c_void_p, C.c_int32, C.c_void_p]
        l.fxp_kv_packed_bytes.restype = C.c_size_t
        l.fxp_kv_packed_bytes.argtypes = [C.POINTER(StageDesc), C.c_int32, C.c_int32, C.c_void_p, C.c_int32]
        l.fxp_kv_pack.argtypes = [C.POINTER(StageDesc), C.POINTER(KvView), C.c_int32, C.c_int32, C.c_void_p,
                                  C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]
        l.fxp_kv_unpack.argtypes = [C.POINTER(StageDesc), C.c_void_p, C.c_size_t, C.POINTER(KvView), C.c_int32,
                                    C.c_int32, C.c_void_p, C.c_int32, C.c_void_p]
        l.fxp_kv_repartition_range.argtypes = [C.POINTER(StageDesc), C.POINTER(KvView), C.c_int32, C.POINTER(KvView),
                                               C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
        l.fxp_kv_packed_tokens_bytes.restype = C.c_size_t
        l.fxp_kv_packed_tokens_bytes.argtypes = [C.POINTER(StageDesc), C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32]
        l.fxp_kv_pack_tokens.argtypes = [C.POINTER(StageDesc), C.POINTER(KvView), C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                         C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]
        l.fxp_kv_unpack_tokens.argtypes = [C.POINTER(StageDesc), C.c_void_p, C.c_size_t, C.POINTER(KvView), C.c_int32,
                                           C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
        l.fxp_ctl_cv.argtypes = [C.POINTER(C.c_double), C.c_int32, C.POINTER(C.c_double)]
        l.fxp_ctl_select_granularity.argtypes = [C.POINTER(Granularity), C.c_int32, C.c_double, C.c_double, C.c_double,
                                                 C.POINTER(C.c_double), C.POINTER(C.c_int32)]
        l.fxp_ctl_parallel_instances.restype = C.c_int64
        l.fxp_ctl_parallel_instances.argtypes = [C.c_double, C.c_double, C.c_double, C.c_double, C.c_int32]
        l.fxp_ctl_multiplexing_penalty.restype = C.c_double
        l.fxp_ctl_multiplexing_penalty.argtypes = [C.c_double, C.c_double, C.c_double]
        l.fxp_ctl_scaling_granularity.restype = C.c_int32
        l.fxp_ctl_scaling_granularity.argtypes = [C.c_int32, C.c_double, C.c_double, C.c_double, C.c_double, C.c_double]
        l.fxp_ctl_slo_satisfied.argtypes = [C.c_double, C.c_double, C.POINTER(C.c_double), C.c_int32, C.c_double, C.c_double]
        l.fxp_profile_class_name.restype = C.c_char_p
        l.fxp_profile_class_name.argtypes = [C.c_int]
        l.fxp_profile_read.argtypes = [C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        l.fxp_profile_read_launch.argtypes = [C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_double)]
        _lib = l
    return _lib


def profile_enable(on: bool) -> None:
    _check(lib().fxp_profile_enable(1 if on else 0))


def profile_launches() -> List[tuple]:
    """[(kernel class name, ms)] of every recorded launch, in launch order."""
    out, i = [], 0
    cls, ms = C.c_int(), C.c_double()
    while lib().fxp_profile_read_launch(i, C.byref(cls), C.byref(ms)) == FXP_OK:
        out.append((lib().fxp_profile_class_name(cls.value).decode(), ms.value))
        i += 1
    return out


def profile_read() -> Dict[str, Dict[str, float]]:
    """{kernel class name: {"ms": summed duration, "launches": count}} for the launches recorded so far."""
    out = {}
    for k in range(lib().fxp_profile_num_classes()):
        ms, n = C.c_double(), C.c_int64()
        _check(lib().fxp_profile_read(k, C.byref(ms), C.byref(n)))
        if n.value:
            out[lib().fxp_profile_class_name(k).decode()] = {"ms": ms.value, "launches": n.value}
    return out


def _check(rc: int) -> None:
    if rc != FXP_OK:
        raise FxpError(rc, lib().fxp_last_error().decode())


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def make_desc(shape, layer_begin: int, layer_end: int) -> StageDesc:
    """``shape`` is any object with hidden / n_q_heads / n_kv_heads / head_dim / ffn /
    rms_eps / rope_base / kv_block_size attributes."""
    return StageDesc(layer_begin, layer_end, shape.hidden, shape.n_q_heads, shape.n_kv_heads,
                     shape.head_dim, shape.ffn, shape.rms_eps, shape.rope_base, shape.kv_block_size,
                     int(getattr(shape, "arch", ARCH_LLAMA)))


@dataclass
class KVCache:
    """A stage's paged cache: ``pool`` is a bf16/int16 CUDA tensor of logical shape
    [layers][blocks][2][Hkv][16][D]; ``block_table`` int32 CUDA [num_seqs][max_blocks]."""
    pool: torch.Tensor
    layer_begin: int
    layer_end: int
    block_table: torch.Tensor

    def c_pool(self) -> KvPool:
        assert self.pool.is_cuda and self.pool.is_contiguous() and self.pool.element_size() == 2
        assert self.pool.shape[0] == self.layer_end - self.layer_begin
        return KvPool(self.pool.data_ptr(), self.pool.shape[1], self.layer_begin, self.layer_end)

    def c_view(self, keep: list) -> KvView:
        assert self.block_table.is_cuda and self.block_table.dtype == torch.int32 and self.block_table.is_contiguous()
        p = self.c_pool(); keep.append(p)
        return KvView(C.pointer(p), self.block_table.data_ptr(), self.block_table.shape[1])


class Stage:
    """fxp_stage_create / fxp_stage_forward / fxp_stage_destroy."""

    def __init__(self, shape, layer_begin: int, layer_end: int, layers: Sequence[Dict[str, torch.Tensor]]):
        self.shape = shape
        self.desc = make_desc(shape, layer_begin, layer_end)
        n = layer_end - layer_begin
        if len(layers) != n:
            raise ValueError("one weight dict per layer")
        arr = (LayerWeights * n)()
        opt = self.desc.arch == ARCH_OPT
        for k, lw in enumerate(layers):
            # Llama-style: the nine fields by name; OPT-style: the sixteen tensors by their usual names
            fields = OPT_TENSOR_FIELDS if opt else {n: n for n in LAYER_TENSORS}
            for name, field in fields.items():
                t = lw[name]
                assert t.is_cuda and t.is_contiguous() and t.element_size() == 2, name
                setattr(arr[k], field, t.data_ptr())
        nbytes = lib().fxp_stage_weight_arena_bytes(C.byref(self.desc))
        if nbytes == 0:
            raise FxpError(FXP_EINVAL, lib().fxp_last_error().decode())
        self.arena = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        handle = C.c_void_p()
        _check(lib().fxp_stage_create(C.byref(self.desc), arr, self.arena.data_ptr(), nbytes, _stream(), C.byref(handle)))
        self.handle = handle
        self._ws: Optional[torch.Tensor] = None

    @classmethod
    def _adopt(cls, shape, handle: C.c_void_p, arena: torch.Tensor) -> "Stage":
        """Wrap a handle made by fxp_stage_split / fxp_stage_merge; ``arena`` is kept alive with it."""
        st = cls.__new__(cls)
        lb, le = C.c_int32(), C.c_int32()
        _check(lib().fxp_stage_layers(handle, C.byref(lb), C.byref(le)))
        st.shape, st.desc, st.arena, st.handle, st._ws = shape, make_desc(shape, lb.value, le.value), arena, handle, None
        return st

    @property
    def layers(self):
        return self.desc.layer_begin, self.desc.layer_end

    def split(self, layer_mid: int):
        """fxp_stage_split: two stages over [begin, mid) and [mid, end) sharing this stage's arena."""
        lo, hi = C.c_void_p(), C.c_void_p()
        _check(lib().fxp_stage_split(self.handle, layer_mid, C.byref(lo), C.byref(hi)))
        return Stage._adopt(self.shape, lo, self.arena), Stage._adopt(self.shape, hi, self.arena)

    def merge(self, upper: "Stage") -> "Stage":
        """fxp_stage_merge: one stage over both ranges; the records must be adjacent in one arena."""
        out = C.c_void_p()
        _check(lib().fxp_stage_merge(self.handle, upper.handle, C.byref(out)))
        return Stage._adopt(self.shape, out, self.arena)

    def close(self) -> None:
        if getattr(self, "handle", None):
            lib().fxp_stage_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def workspace_bytes(self, max_tokens: int, max_seqs: int, max_blocks_per_seq: int) -> int:
        return lib().fxp_stage_workspace_bytes(self.handle, max_tokens, max_seqs, max_blocks_per_seq)

    def _workspace(self, nbytes: int) -> torch.Tensor:
        if self._ws is None or self._ws.numel() < nbytes:
            self._ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        return self._ws

    def forward(self, cache: KVCache, cu_seqlens_q: torch.Tensor, ctx_lens: torch.Tensor, hidden_in: torch.Tensor,
                max_q_len: int, hidden_out: Optional[torch.Tensor] = None,
                probs: Optional[torch.Tensor] = None, min_q_len: int = 0) -> torch.Tensor:
        """One step.  ``hidden_in`` bf16 CUDA [T,H]; ``cu_seqlens_q`` int32 CUDA [B+1]; ``ctx_lens`` int32 CUDA [B].
        ``probs`` (float32 CUDA [layers][T][Hq][stride]) switches to the debug entry point.  ``min_q_len`` is the
        optional hint of the ABI (0 = not known)."""
        T = hidden_in.shape[0]
        B = ctx_lens.shape[0]
        assert hidden_in.is_cuda and hidden_in.is_contiguous() and hidden_in.element_size() == 2
        assert cu_seqlens_q.dtype == torch.int32 and ctx_lens.dtype == torch.int32
        if hidden_out is None:
            hidden_out = torch.empty_like(hidden_in)
        pool = cache.c_pool()
        batch = Batch(B, T, max_q_len, cache.block_table.shape[1], cu_seqlens_q.data_ptr(), ctx_lens.data_ptr(),
                      cache.block_table.data_ptr(), min_q_len)
        nbytes = self.workspace_bytes(T, B, cache.block_table.shape[1])
        ws = self._workspace(nbytes)
        if probs is None:
            _check(lib().fxp_stage_forward(self.handle, C.byref(pool), C.byref(batch), hidden_in.data_ptr(),
                                           hidden_out.data_ptr(), ws.data_ptr(), ws.numel(), _stream()))
        else:
            assert probs.dtype == torch.float32 and probs.is_contiguous()
            _check(lib().fxp_stage_forward_debug(self.handle, C.byref(pool), C.byref(batch), hidden_in.data_ptr(),
                                                 hidden_out.data_ptr(), ws.data_ptr(), ws.numel(), probs.data_ptr(),
                                                 probs.shape[-1], _stream()))
        return hidden_out

    def forward_static(self, cache: KVCache, cu_seqlens_q: torch.Tensor, ctx_lens: torch.Tensor, hidden_in: torch.Tensor,
                       max_q_len: int, hidden_out: torch.Tensor, min_q_len: int = 0) -> torch.Tensor:
        """fxp_stage_forward_static: the same step with the library's static scratch as workspace; the caller
        passes the output buffer too, so nothing is allocated on this path."""
        T, B = hidden_in.shape[0], ctx_lens.shape[0]
        assert hidden_in.is_cuda and hidden_in.is_contiguous() and hidden_in.element_size() == 2
        assert hidden_out.is_cuda and hidden_out.is_contiguous() and hidden_out.shape == hidden_in.shape
        assert cu_seqlens_q.dtype == torch.int32 and ctx_lens.dtype == torch.int32
        pool = cache.c_pool()
        batch = Batch(B, T, max_q_len, cache.block_table.shape[1], cu_seqlens_q.data_ptr(), ctx_lens.data_ptr(),
                      cache.block_table.data_ptr(), min_q_len)
        _check(lib().fxp_stage_forward_static(self.handle, C.byref(pool), C.byref(batch), hidden_in.data_ptr(),
                                              hidden_out.data_ptr(), _stream()))
        return hidden_out


def kv_repartition(shape, src: Sequence[KVCache], dst: Sequence[KVCache], ctx_lens: torch.Tensor) -> None:
    keep: list = []
    desc = make_desc(shape, 0, 1)
    s = (KvView * len(src))(*[v.c_view(keep) for v in src])
    d = (KvView * len(dst))(*[v.c_view(keep) for v in dst])
    assert ctx_lens.is_cuda and ctx_lens.dtype == torch.int32
    _check(lib().fxp_kv_repartition(C.byref(desc), s, len(src), d, len(dst), ctx_lens.data_ptr(), ctx_lens.shape[0], _stream()))


def kv_packed_bytes(shape, layer_begin: int, layer_end: int, ctx_lens_host) -> int:
    import numpy as np
    cl = np.ascontiguousarray(ctx_lens_host, dtype=np.int32)
    desc = make_desc(shape, 0, 1)
    return lib().fxp_kv_packed_bytes(C.byref(desc), layer_begin, layer_end, cl.ctypes.data, cl.shape[0])


def kv_pack(shape, src: KVCache, layer_begin: int, layer_end: int, ctx_lens: torch.Tensor, packed: torch.Tensor) -> None:
    keep: list = []
    desc = make_desc(shape, 0, 1)
    v = src.c_view(keep)
    _check(lib().fxp_kv_pack(C.byref(desc), C.byref(v), layer_begin, layer_end, ctx_lens.data_ptr(), ctx_lens.shape[0],
                             packed.data_ptr(), packed.numel() * packed.element_size(), _stream()))


def kv_unpack(shape, packed: torch.Tensor, dst: KVCache, layer_begin: int, layer_end: int, ctx_lens: torch.Tensor) -> None:
    keep: list = []
    desc = make_desc(shape, 0, 1)
    v = dst.c_view(keep)
    _check(lib().fxp_kv_unpack(C.byref(desc), packed.data_ptr(), packed.numel() * packed.element_size(), C.byref(v),
                               layer_begin, layer_end, ctx_lens.data_ptr(), ctx_lens.shape[0], _stream()))


def _lens_ptr(t: torch.Tensor) -> int:
    assert t.is_cuda and t.dtype == torch.int32 and t.is_contiguous()
    return t.data_ptr()


def kv_repartition_range(shape, src: Sequence[KVCache], dst: Sequence[KVCache], from_lens: torch.Tensor,
                         to_lens: torch.Tensor) -> None:
    """Incremental pass: only tokens [from_lens[i], to_lens[i]) of every sequence."""
    keep: list = []
    desc = make_desc(shape, 0, 1)
    s = (KvView * len(src))(*[v.c_view(keep) for v in src])
    d = (KvView * len(dst))(*[v.c_view(keep) for v in dst])
    assert from_lens.shape == to_lens.shape
    _check(lib().fxp_kv_repartition_range(C.byref(desc), s, len(src), d, len(dst), _lens_ptr(from_lens), _lens_ptr(to_lens),
                                          to_lens.shape[0], _stream()))


def kv_packed_tokens_bytes(shape, layer_begin: int, layer_end: int, from_lens_host, to_lens_host) -> int:
    import numpy as np
    fl = np.ascontiguousarray(from_lens_host, dtype=np.int32)
    tl = np.ascontiguousarray(to_lens_host, dtype=np.int32)
    assert fl.shape == tl.shape
    desc = make_desc(shape, 0, 1)
    return lib().fxp_kv_packed_tokens_bytes(C.byref(desc), layer_begin, layer_end, fl.ctypes.data, tl.ctypes.data, tl.shape[0])


def kv_pack_tokens(shape, src: KVCache, layer_begin: int, layer_end: int, from_lens: torch.Tensor, to_lens: torch.Tensor,
                   packed: torch.Tensor) -> None:
    keep: list = []
    desc = make_desc(shape, 0, 1)
    v = src.c_view(keep)
    _check(lib().fxp_kv_pack_tokens(C.byref(desc), C.byref(v), layer_begin, layer_end, _lens_ptr(from_lens), _lens_ptr(to_lens),
                                    to_lens.shape[0], packed.data_ptr(), packed.numel() * packed.element_size(), _stream()))


def kv_unpack_tokens(shape, packed: torch.Tensor, dst: KVCache, layer_begin: int, layer_end: int, from_lens: torch.Tensor,
                     to_lens: torch.Tensor) -> None:
    keep: list = []
    desc = make_desc(shape, 0, 1)
    v = dst.c_view(keep)
    _check(lib().fxp_kv_unpack_tokens(C.byref(desc), packed.data_ptr(), packed.numel() * packed.element_size(), C.byref(v),
                                      layer_begin, layer_end, _lens_ptr(from_lens), _lens_ptr(to_lens), to_lens.shape[0],
                                      _stream()))


# ---- granularity controller (host only) ------------------------------------------------

def ctl_cv(intervals) -> float:
    arr = (C.c_double * len(intervals))(*[float(v) for v in intervals])
    out = C.c_double()
    _check(lib().fxp_ctl_cv(arr, len(intervals), C.byref(out)))
    return out.value


def ctl_select_granularity(cands: Sequence[Granularity], cv_now: float, alpha: float, sigma: float):
    """Eq. 4: returns (index of the best candidate, list of scores)."""
    arr = (Granularity * len(cands))(*cands)
    scores = (C.c_double * len(cands))()
    best = C.c_int32()
    _check(lib().fxp_ctl_select_granularity(arr, len(cands), cv_now, alpha, sigma, scores, C.byref(best)))
    return best.value, list(scores)


def ctl_parallel_instances(capacity_total: float, throughput: float, beta1: float, beta2: float, n_stages: int) -> int:
    r = lib().fxp_ctl_parallel_instances(capacity_total, throughput, beta1, beta2, n_stages)
    if r < 0:
        raise FxpError(FXP_EINVAL, lib().fxp_last_error().decode())
    return r


def ctl_multiplexing_penalty(gamma0: float, alpha: float, cv: float) -> float:
    return lib().fxp_ctl_multiplexing_penalty(gamma0, alpha, cv)


def ctl_scaling_granularity(g_max: int, beta: float, gamma: float, cv: float, queue_len: float, queue_cap: float) -> int:
    r = lib().fxp_ctl_scaling_granularity(g_max, beta, gamma, cv, queue_len, queue_cap)
    if r < 0:
        raise FxpError(FXP_EINVAL, lib().fxp_last_error().decode())
    return r


def ctl_slo_satisfied(deadline: float, init_time: float, stage_throughput, queue_len: float, requests: float) -> bool:
    arr = (C.c_double * len(stage_throughput))(*[float(v) for v in stage_throughput])
    r = lib().fxp_ctl_slo_satisfied(deadline, init_time, arr, len(stage_throughput), queue_len, requests)
    if r < 0:
        raise FxpError(r, lib().fxp_last_error().decode())
    return bool(r)
