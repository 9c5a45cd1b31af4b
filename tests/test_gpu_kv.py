"""GPU parity for KV repartition / pack / unpack (Section 6.3, Eq. 10): the HIP
path must equal the oracle bit for bit on the 16-bit words, including the
zeroed invalid slots and the untouched blocks."""
import numpy as np
import pytest
import torch

import oracle
from oracle import KVView
from paper_2510_11938_amd import binding, synth

from gpu_util import dev_i32, host_bits, oracle_shape

pytestmark = pytest.mark.gpu


def geom(hkv, d):
    return synth.ModelShape(hidden=hkv * d, n_q_heads=hkv, n_kv_heads=hkv, head_dim=d, ffn=64)


def make_views(ms, ranges, lens, seed, spare=2):
    """Host views with random junk everywhere + device copies."""
    rng = np.random.default_rng(seed)
    host, dev = [], []
    for s, (a, b) in enumerate(ranges):
        table, nblk = synth.block_table(lens, ms.kv_block_size, seed=seed, salt=20 + s, spare_blocks=spare)
        pool = rng.integers(1, 65536, size=(b - a, nblk, 2, ms.n_kv_heads, 16, ms.head_dim), dtype=np.uint16)
        host.append(KVView(pool, a, b, table))
        dev.append(binding.KVCache(torch.from_numpy(pool.view(np.int16)).cuda(), a, b, dev_i32(table)))
    return host, dev


CASES = [
    # (Hkv, D, src ranges, dst ranges, lengths)
    (4, 64, [(0, 2)], [(0, 1), (1, 2)], [37, 128, 32, 100]),                      # tiny config: split
    (4, 64, [(0, 1), (1, 2)], [(0, 2)], [37, 128, 32, 100]),                      # tiny config: merge
    (2, 8, [(3, 5), (5, 9)], [(3, 6), (6, 7), (7, 9)], [5, 16, 1, 0, 11, 250]),   # 512-byte units, empty sequence
    (3, 128, [(0, 3)], [(0, 1), (1, 3)], [300, 17, 64]),                          # 24 KiB units: ragged last chunk
    (1, 64, [(0, 2)], [(0, 2)], [1, 15, 16, 17]),                                 # 4 KiB units, same ranges, new table
    (8, 128, [(0, 4)], [(0, 2), (2, 4)], [1024, 333, 2047, 16, 700, 1, 1500, 96]),  # 64 KiB units (70B shape)
    (32, 128, [(0, 2)], [(0, 1), (1, 2)], [200, 513]),                            # 256 KiB units (7B shape)
]


@pytest.mark.parametrize("hkv,d,src_r,dst_r,lens", CASES)
def test_repartition_matches_oracle_bit_exact(hkv, d, src_r, dst_r, lens):
    ms = geom(hkv, d)
    lens = np.array(lens, dtype=np.int32)
    hs, ds = make_views(ms, src_r, lens, seed=1)
    hd, dd = make_views(ms, dst_r, lens, seed=2, spare=3)
    oracle.kv_repartition(oracle_shape(ms), hs, hd, lens)
    binding.kv_repartition(ms, ds, dd, dev_i32(lens))
    torch.cuda.synchronize()
    for h, g in zip(hd, dd):
        assert np.array_equal(host_bits(g.pool), h.pool)
    for h, g in zip(hs, ds):                                  # sources untouched
        assert np.array_equal(host_bits(g.pool), h.pool)


def test_repartition_with_more_than_eight_jobs():
    ms = geom(2, 64)
    lens = np.array([40, 7, 90], dtype=np.int32)
    src_r = [(i, i + 1) for i in range(12)]
    dst_r = [(0, 5), (5, 12)]
    hs, ds = make_views(ms, src_r, lens, seed=3)
    hd, dd = make_views(ms, dst_r, lens, seed=4)
    oracle.kv_repartition(oracle_shape(ms), hs, hd, lens)
    binding.kv_repartition(ms, ds, dd, dev_i32(lens))
    torch.cuda.synchronize()
    for h, g in zip(hd, dd):
        assert np.array_equal(host_bits(g.pool), h.pool)


def test_split_then_merge_round_trip_on_gpu():
    ms = geom(4, 64)
    lens = synth.draw_lengths(("uniform", 32, 128), 4, seed=0)
    _, a = make_views(ms, [(0, 2)], lens, seed=5)
    _, b = make_views(ms, [(0, 1), (1, 2)], lens, seed=6)
    c = [binding.KVCache(torch.zeros_like(a[0].pool), 0, 2, a[0].block_table.clone())]
    cl = dev_i32(lens)
    binding.kv_repartition(ms, a, b, cl)
    binding.kv_repartition(ms, b, c, cl)
    torch.cuda.synchronize()
    pa, pc, table = host_bits(a[0].pool), host_bits(c[0].pool), a[0].block_table.cpu().numpy()
    for i, n in enumerate(lens):
        for j in range((n + 15) // 16):
            v = min(16, n - 16 * j)
            assert np.array_equal(pc[:, table[i, j], :, :, :v], pa[:, table[i, j], :, :, :v])
            assert np.all(pc[:, table[i, j], :, :, v:] == 0)


@pytest.mark.parametrize("hkv,d,lens", [(4, 64, [37, 0, 128, 5]), (3, 128, [300, 17]), (8, 128, [1000, 2047, 1])])
def test_pack_and_unpack_match_oracle(hkv, d, lens):
    ms = geom(hkv, d)
    osh = oracle_shape(ms)
    lens = np.array(lens, dtype=np.int32)
    hs, ds = make_views(ms, [(2, 6)], lens, seed=7)
    lb, le = 3, 6
    want = oracle.kv_pack(osh, hs[0], lb, le, lens)
    nbytes = binding.kv_packed_bytes(ms, lb, le, lens)
    assert nbytes == want.size * 2
    packed = torch.full((nbytes // 2,), 0x5555, dtype=torch.int16, device="cuda")
    cl = dev_i32(lens)
    binding.kv_pack(ms, ds[0], lb, le, cl, packed)
    torch.cuda.synchronize()
    assert np.array_equal(host_bits(packed), want)
    hd, dd = make_views(ms, [(3, 6)], lens, seed=8, spare=1)
    oracle.kv_unpack(osh, want, hd[0], lb, le, lens)
    binding.kv_unpack(ms, packed, dd[0], lb, le, cl)
    torch.cuda.synchronize()
    assert np.array_equal(host_bits(dd[0].pool), hd[0].pool)


def test_pack_never_writes_past_a_short_buffer():
    ms = geom(4, 64)
    lens = np.array([64, 64], dtype=np.int32)
    _, ds = make_views(ms, [(0, 1)], lens, seed=9)
    unit = ms.block_elems                                    # int16 elements per (layer, block)
    guard = torch.full((8 * unit + 4096,), 0x7777, dtype=torch.int16, device="cuda")
    short = guard[: 5 * unit]                                # room for 5 of the 8 blocks
    binding.kv_pack(ms, ds[0], 0, 1, dev_i32(lens), short)
    torch.cuda.synchronize()
    assert bool((guard[5 * unit:] == 0x7777).all())


def test_argument_errors_are_reported_not_launched():
    ms = geom(4, 64)
    lens = np.array([10], dtype=np.int32)
    _, a = make_views(ms, [(0, 2)], lens, seed=10)
    _, b = make_views(ms, [(0, 1), (2, 3)], lens, seed=11)
    with pytest.raises(binding.FxpError) as e:
        binding.kv_repartition(ms, a, b, dev_i32(lens))
    assert e.value.code == binding.FXP_EINVAL
    with pytest.raises(binding.FxpError):                    # overlapping source and destination
        binding.kv_repartition(ms, a, a, dev_i32(lens))
    binding.kv_repartition(ms, a, [binding.KVCache(torch.zeros_like(a[0].pool), 0, 2, a[0].block_table)],
                           torch.zeros(0, dtype=torch.int32, device="cuda"))     # zero sequences: no-op


def test_full_size_7b_repartition_sampled_against_oracle():
    """The benchmark's repartition (7B shape, 4 layers -> 2 + 2, B = 32, contexts
    U[512,4096]) at full size.  All blocks are checked with an independent torch
    gather through both tables; four sampled sequences are also checked against
    the oracle, which moves only those."""
    wl = synth.WORKLOADS["C2"]
    ms = wl.shape
    lens = synth.draw_lengths(wl.length_dist, wl.num_seqs, wl.seed)
    t_src, n_src = synth.block_table(lens + 1, 16, wl.seed, salt=0)
    g = torch.Generator(device="cuda"); g.manual_seed(7)
    src_pool = torch.randint(-32768, 32767, (4, n_src, 2, ms.n_kv_heads, 16, ms.head_dim), dtype=torch.int16,
                             device="cuda", generator=g)
    src = [binding.KVCache(src_pool, 0, 4, dev_i32(t_src))]
    dst = []
    for s, (a, b) in enumerate([(0, 2), (2, 4)]):
        t, n = synth.block_table(lens + 1, 16, wl.seed, salt=1 + s)
        dst.append(binding.KVCache(torch.full((b - a, n, 2, ms.n_kv_heads, 16, ms.head_dim), 0x1111, dtype=torch.int16,
                                              device="cuda"), a, b, dev_i32(t)))
    binding.kv_repartition(ms, src, dst, dev_i32(lens))
    torch.cuda.synchronize()
    nblk = (lens + 15) // 16
    for dv in dst:
        owned = torch.zeros(dv.pool.shape[1], dtype=torch.bool, device="cuda")
        for i in range(wl.num_seqs):
            sb = src[0].block_table[i, : nblk[i]].long(); db = dv.block_table[i, : nblk[i]].long()
            owned[db] = True
            got = dv.pool[:, db]                                           # [layers][blocks][2][H][16][D]
            want = src_pool[dv.layer_begin:dv.layer_end][:, sb].clone()
            tail = int(lens[i] % 16)
            if tail:
                want[:, -1, :, :, tail:, :] = 0
            assert torch.equal(got, want), f"sequence {i}"
        assert bool((dv.pool[:, ~owned] == 0x1111).all())
    # oracle on a sample of sequences (others given length 0)
    sample = [0, 7, 19, 31]
    sub = np.zeros_like(lens); sub[sample] = lens[sample]
    osh = oracle_shape(ms)
    hs = [KVView(host_bits(src_pool), 0, 4, t_src)]
    for dv in dst:
        hp = np.full(tuple(dv.pool.shape), 0x1111, dtype=np.uint16)
        oracle.kv_repartition(osh, [KVView(hs[0].pool[dv.layer_begin:dv.layer_end].copy(), dv.layer_begin, dv.layer_end, t_src)],
                              [KVView(hp, dv.layer_begin, dv.layer_end, dv.block_table.cpu().numpy())], sub)
        gp = host_bits(dv.pool)
        for i in sample:
            blocks = dv.block_table[i, : nblk[i]].cpu().numpy()
            assert np.array_equal(gp[:, blocks], hp[:, blocks])


# ---------------------------------------------------------------------------
# Incremental passes (Section 6.3: the transfer runs while decoding continues) and
# the token-dense packed form: same bit-exact bar against the oracle.

RANGE_CASES = [
    # (Hkv, D, src ranges, dst ranges, from, to)
    (4, 64, [(0, 2)], [(0, 1), (1, 2)], [30, 128, 0, 100], [37, 128, 32, 117]),                # none / zero-length / from empty / crosses a block
    (2, 8, [(3, 5), (5, 9)], [(3, 6), (6, 7), (7, 9)], [5, 16, 1, 0, 11, 250], [6, 17, 1, 0, 40, 251]),
    (3, 128, [(0, 3)], [(0, 1), (1, 3)], [299, 0, 63], [300, 17, 97]),                         # 24 KiB units
    (8, 128, [(0, 4)], [(0, 2), (2, 4)], [1000, 333, 2047, 16, 0], [1024, 334, 2050, 16, 700]),  # 64 KiB units
    (32, 128, [(0, 2)], [(0, 1), (1, 2)], [199, 512], [200, 530]),                             # 256 KiB units (7B shape)
]


@pytest.mark.parametrize("hkv,d,src_r,dst_r,lo,hi", RANGE_CASES)
def test_range_repartition_matches_oracle_bit_exact(hkv, d, src_r, dst_r, lo, hi):
    ms = geom(hkv, d)
    lo, hi = np.array(lo, dtype=np.int32), np.array(hi, dtype=np.int32)
    hs, ds = make_views(ms, src_r, hi, seed=11)
    hd, dd = make_views(ms, dst_r, hi, seed=12, spare=3)
    oracle.kv_repartition_range(oracle_shape(ms), hs, hd, lo, hi)
    binding.kv_repartition_range(ms, ds, dd, dev_i32(lo), dev_i32(hi))
    torch.cuda.synchronize()
    for h, g in zip(hd, dd):
        assert np.array_equal(host_bits(g.pool), h.pool)          # moved rows, zeroed tail, everything else untouched
    for h, g in zip(hs, ds):
        assert np.array_equal(host_bits(g.pool), h.pool)


def test_snapshot_pass_then_delta_pass_equals_one_pass_on_gpu():
    ms = geom(4, 64)
    snap = np.array([37, 128, 0, 100, 15], dtype=np.int32)
    now = np.array([40, 128, 5, 117, 16], dtype=np.int32)
    _, src = make_views(ms, [(0, 1), (1, 3)], now, seed=13)
    _, one = make_views(ms, [(0, 3)], now, seed=14)
    _, two = make_views(ms, [(0, 3)], now, seed=14)
    binding.kv_repartition(ms, src, one, dev_i32(now))
    binding.kv_repartition(ms, src, two, dev_i32(snap))
    binding.kv_repartition_range(ms, src, two, dev_i32(snap), dev_i32(now))
    torch.cuda.synchronize()
    assert np.array_equal(host_bits(one[0].pool), host_bits(two[0].pool))


def test_range_with_inverted_or_negative_range_moves_nothing_for_that_sequence():
    ms = geom(2, 64)
    hi = np.array([20, 20, 20], dtype=np.int32)
    lo = np.array([25, -3, 4], dtype=np.int32)                    # the library reads lengths on the device: it cannot reject these
    hs, ds = make_views(ms, [(0, 1)], hi, seed=15)
    hd, dd = make_views(ms, [(0, 1)], hi, seed=16)
    ok_lo, ok_hi = np.array([0, 0, 4], dtype=np.int32), np.array([0, 0, 20], dtype=np.int32)
    oracle.kv_repartition_range(oracle_shape(ms), hs, hd, ok_lo, ok_hi)     # what must happen: only sequence 2 moves
    binding.kv_repartition_range(ms, ds, dd, dev_i32(lo), dev_i32(hi))
    torch.cuda.synchronize()
    assert np.array_equal(host_bits(dd[0].pool), hd[0].pool)


@pytest.mark.parametrize("hkv,d,lo,hi", [(4, 64, [30, 0, 128, 5, 9], [37, 0, 128, 40, 10]), (3, 128, [0, 16], [300, 17]),
                                          (8, 128, [990, 2047, 0], [1000, 2050, 1])])
def test_token_dense_pack_and_unpack_match_oracle(hkv, d, lo, hi):
    ms = geom(hkv, d)
    osh = oracle_shape(ms)
    lo, hi = np.array(lo, dtype=np.int32), np.array(hi, dtype=np.int32)
    hs, ds = make_views(ms, [(2, 6)], hi, seed=17)
    lb, le = 3, 6
    want = oracle.kv_pack_tokens(osh, hs[0], lb, le, lo, hi)
    nbytes = binding.kv_packed_tokens_bytes(ms, lb, le, lo, hi)
    assert nbytes == want.size * 2
    pad = 64                                                       # guard words after the buffer must survive
    packed = torch.full((nbytes // 2 + pad,), 0x5555, dtype=torch.int16, device="cuda")
    dlo, dhi = dev_i32(lo), dev_i32(hi)
    binding.kv_pack_tokens(ms, ds[0], lb, le, dlo, dhi, packed[:nbytes // 2])
    torch.cuda.synchronize()
    got = host_bits(packed)
    assert np.array_equal(got[:nbytes // 2], want)
    assert np.all(got[nbytes // 2:] == 0x5555)
    hd, dd = make_views(ms, [(3, 6)], hi, seed=18, spare=1)
    oracle.kv_unpack_tokens(osh, want, hd[0], lb, le, lo, hi)
    binding.kv_unpack_tokens(ms, packed[:nbytes // 2], dd[0], lb, le, dlo, dhi)
    torch.cuda.synchronize()
    assert np.array_equal(host_bits(dd[0].pool), hd[0].pool)


def test_token_dense_pack_never_writes_past_a_short_buffer():
    ms = geom(4, 64)
    lo, hi = np.array([0, 3], dtype=np.int32), np.array([50, 40], dtype=np.int32)
    hs, ds = make_views(ms, [(0, 2)], hi, seed=19)
    want = oracle.kv_pack_tokens(oracle_shape(ms), hs[0], 0, 2, lo, hi)
    short = want.size // 3 // 8 * 8                                # a third of the needed size, whole 16-byte vectors
    packed = torch.full((want.size,), 0x5555, dtype=torch.int16, device="cuda")
    binding.kv_pack_tokens(ms, ds[0], 0, 2, dev_i32(lo), dev_i32(hi), packed[:short])
    torch.cuda.synchronize()
    got = host_bits(packed)
    assert np.array_equal(got[:short], want[:short])               # what fits is right
    assert np.all(got[short:] == 0x5555)                           # nothing beyond the size given


def test_repartition_with_the_maximum_number_of_sequences():
    """FXP_MAX_SEQS sequences (the per-workgroup prefix scans at their largest), many of them empty."""
    ms = geom(2, 8)
    rng = np.random.default_rng(31)
    lens = rng.integers(0, 40, size=4096).astype(np.int32)
    lens[rng.integers(0, 4096, size=500)] = 0
    hs, ds = make_views(ms, [(0, 2)], lens, seed=32)
    hd, dd = make_views(ms, [(0, 1), (1, 2)], lens, seed=33)
    oracle.kv_repartition(oracle_shape(ms), hs, hd, lens)
    binding.kv_repartition(ms, ds, dd, dev_i32(lens))
    torch.cuda.synchronize()
    for h, g in zip(hd, dd):
        assert np.array_equal(host_bits(g.pool), h.pool)
    with pytest.raises(binding.FxpError):
        binding.kv_repartition(ms, ds, dd, dev_i32(np.zeros(4097, dtype=np.int32)))
