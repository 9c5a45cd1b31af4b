"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every function the public header declares, and its argument validation returns
error codes (never launches) for malformed calls."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2510_11938_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "flexstage.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fxp_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    lib = binding.lib()
    for n in names:
        assert hasattr(lib, n), n
    assert b"gfx950" in lib.fxp_version()


def test_arena_and_packed_sizes_are_host_computations():
    lib = binding.lib()
    ms = synth.LLAMA2_7B
    d = binding.make_desc(ms, 0, 4)
    # per layer: every matrix re-tiled with k padded to 64, plus the two gains
    per_layer = 2 * (ms.qkv_out * 4096 + 4096 * 4096 + 2 * 11008 * 4096 + 4096 * 11008) + 2 * 4096 * 2
    assert lib.fxp_stage_weight_arena_bytes(C.byref(d)) == 4 * per_layer
    # ffn 688 is padded to 704 as the k of the down projection; the 1376 gate|up rows take whole groups of 8 x 16 rows (1408)
    tiny = binding.make_desc(synth.TINY, 0, 1)
    assert lib.fxp_stage_weight_arena_bytes(C.byref(tiny)) == 2 * (768 * 256 + 256 * 256 + 1408 * 256 + 256 * 704) + 2 * 512
    lens = np.array([1, 16, 17, 0, 4096], dtype=np.int32)
    assert binding.kv_packed_bytes(ms, 2, 4, lens) == (1 + 1 + 2 + 0 + 256) * 2 * (2 * 32 * 16 * 128 * 2)


@pytest.mark.parametrize("field,value", [("kv_block_size", 32), ("head_dim", 96), ("n_kv_heads", 3), ("hidden", 100),
                                         ("ffn", 0), ("layer_end", 0)])
def test_bad_descriptors_are_rejected(field, value):
    lib = binding.lib()
    d = binding.make_desc(synth.TINY, 0, 2)
    setattr(d, field, value)
    assert lib.fxp_stage_weight_arena_bytes(C.byref(d)) == 0
    assert len(lib.fxp_last_error()) > 0
    out = C.c_void_p()
    w = (binding.LayerWeights * 2)()
    assert lib.fxp_stage_create(C.byref(d), w, None, 0, None, C.byref(out)) == binding.FXP_EINVAL


def test_null_and_malformed_repartition_arguments():
    lib = binding.lib()
    d = binding.make_desc(synth.TINY, 0, 1)
    assert lib.fxp_kv_repartition(C.byref(d), None, 0, None, 0, None, 0, None) == binding.FXP_EINVAL
    pool_a = binding.KvPool(0x1000, 4, 0, 2)
    pool_b = binding.KvPool(0x9000000, 4, 0, 1)
    va = binding.KvView(C.pointer(pool_a), 0x2000, 4)
    vb = binding.KvView(C.pointer(pool_b), 0x3000, 4)
    # destination does not cover the source's layers
    assert lib.fxp_kv_repartition(C.byref(d), C.byref(va), 1, C.byref(vb), 1, 0x4000, 1, None) == binding.FXP_EINVAL
    assert b"differ" in lib.fxp_last_error()
    # too many sequences for the in-kernel prefix table
    pool_b.layer_end = 2
    assert lib.fxp_kv_repartition(C.byref(d), C.byref(va), 1, C.byref(vb), 1, 0x4000, 1 << 20, None) == binding.FXP_EINVAL
    assert lib.fxp_stage_forward(None, None, None, None, None, None, 0, None) == binding.FXP_EINVAL
    assert lib.fxp_stage_workspace_bytes(None, 1, 1, 1) == 0


def test_split_and_merge_reject_null_handles_without_touching_the_gpu():
    import ctypes as C
    l = binding.lib()
    a, b = C.c_void_p(), C.c_void_p()
    assert l.fxp_stage_split(None, 1, C.byref(a), C.byref(b)) == binding.FXP_EINVAL
    assert l.fxp_stage_merge(None, None, C.byref(a)) == binding.FXP_EINVAL
    lo, hi = C.c_int32(), C.c_int32()
    assert l.fxp_stage_layers(None, C.byref(lo), C.byref(hi)) == binding.FXP_EINVAL
    assert b"null" in l.fxp_last_error()


def test_sequence_count_limit_is_checked_on_the_host():
    """FXP_MAX_SEQS (the per-sequence prefix sums live in LDS): one more is rejected before any launch."""
    import ctypes as C
    l = binding.lib()
    desc = binding.make_desc(synth.TINY, 0, 1)
    pool = binding.KvPool(0x1000, 4, 0, 1)
    view = binding.KvView(C.pointer(pool), 0x2000, 4)
    pool2 = binding.KvPool(0x100000, 4, 0, 1)
    view2 = binding.KvView(C.pointer(pool2), 0x3000, 4)
    rc = l.fxp_kv_repartition(C.byref(desc), C.byref(view), 1, C.byref(view2), 1, 0x4000, 4097, None)
    assert rc == binding.FXP_EINVAL and b"4096" in l.fxp_last_error()
