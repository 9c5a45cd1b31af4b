"""The index arithmetic of the prefill-attention key pieces, restated on the host.

A launch with few query tiles cuts the keys of every tile into up to `kv_split`
pieces (each at least 8 LDS tiles of 64 keys); a piece leaves its partial state
in row `(piece * T + token) * Hq + head` of a buffer whose size depends only on
the token budget of the workspace, and a merge kernel finds the pieces of a row
again from the same lengths.  These tests check what makes that sound, for
random batches: the pieces of a tile cover its key tiles exactly once, none is
shorter than the minimum, every row written lies inside the buffer (also when
the workspace was sized for a larger call), and the merge kernel derives the
same piece count as the attention kernel for every token.  (Pure host
arithmetic; the kernels are checked against the oracle in the GPU tests.)
"""
import numpy as np
import pytest

KV_TILE, MIN_PIECE_TILES, MAX_PIECES, BLOCK = 64, 8, 8, 16


def resident_wgs(q_tile):
    return 768 if q_tile == 64 else 512


def q_tile_of(Hq, T, B, max_q, max_blocks):
    if T < 128 * max(B, 1):
        return 64
    tiles = Hq * (T // 128)
    if tiles >= 768:
        return 128
    prefix_room = max_blocks * BLOCK - max_q >= 2 * MIN_PIECE_TILES * KV_TILE
    return 128 if prefix_room and tiles * MAX_PIECES >= resident_wgs(128) else 64


def piece_rows(Hq, max_tokens):
    return min(max(resident_wgs(64) * 64, resident_wgs(128) * 128), MAX_PIECES * max(max_tokens, 1) * Hq)


def kv_split_of(Hq, T, B, max_blocks, q_tile):
    fits = piece_rows(Hq, T) // (max(T, 1) * Hq)
    if max_blocks * BLOCK < 2 * MIN_PIECE_TILES * KV_TILE:
        return 1
    wgs = Hq * (T // q_tile + B)
    return max(1, min(MAX_PIECES, resident_wgs(q_tile) // wgs, fits))


def kv_pieces(n_tiles, kv_split):
    return min(kv_split, max(1, n_tiles // MIN_PIECE_TILES))


def tile_range(piece, n_pieces, n_tiles):
    return piece * n_tiles // n_pieces, (piece + 1) * n_tiles // n_pieces


def random_batch(rng):
    Hq = int(rng.choice([1, 2, 4, 8, 32, 40, 64]))
    B = int(rng.integers(1, 12))
    q = rng.integers(1, int(rng.choice([8, 100, 700, 3000])), size=B)
    ctx = rng.integers(0, int(rng.choice([1, 300, 5000, 40000])), size=B)
    max_blocks = int((ctx + q + BLOCK - 1).max() // BLOCK) + int(rng.integers(0, 50))
    return Hq, q.astype(np.int64), ctx.astype(np.int64), max_blocks


@pytest.mark.parametrize("seed", range(40))
def test_pieces_cover_every_key_tile_once_and_rows_stay_inside_the_buffer(seed):
    rng = np.random.default_rng(seed)
    Hq, q, ctx, max_blocks = random_batch(rng)
    T, B = int(q.sum()), len(q)
    qt_rows = q_tile_of(Hq, T, B, int(q.max()), max_blocks)
    split = kv_split_of(Hq, T, B, max_blocks, qt_rows)
    assert 1 <= split <= MAX_PIECES
    # the buffer of a workspace sized for a larger call serves this one too
    for budget in (T, T + 1, 4 * T + 100):
        assert split == 1 or split * T * Hq <= piece_rows(Hq, budget)     # uncut tiles write no rows
    cu = np.concatenate([[0], np.cumsum(q)])
    for i in range(B):
        for qt in range((q[i] + qt_rows - 1) // qt_rows):
            wg_last_pos = ctx[i] + min(qt * qt_rows + qt_rows - 1, q[i] - 1)
            n_tiles = wg_last_pos // KV_TILE + 1
            n_pieces = kv_pieces(n_tiles, split)
            covered = []
            for piece in range(n_pieces):
                lo, hi = tile_range(piece, n_pieces, n_tiles)
                assert hi > lo
                if n_pieces > 1:
                    assert hi - lo >= MIN_PIECE_TILES
                covered += list(range(lo, hi))
            assert covered == list(range(n_tiles))
            # the merge kernel, token by token, from the same lengths
            for j in range(qt * qt_rows, min((qt + 1) * qt_rows, q[i])):
                t = cu[i] + j
                qt_m = (t - cu[i]) // qt_rows
                last_m = ctx[i] + min(qt_m * qt_rows + qt_rows - 1, q[i] - 1)
                assert kv_pieces(last_m // KV_TILE + 1, split) == n_pieces
                assert n_pieces == 1 or (n_pieces - 1) * T * Hq + t * Hq + Hq - 1 < piece_rows(Hq, T)


def test_piece_zero_always_holds_the_first_key_so_the_merged_maximum_is_finite():
    for n_tiles in range(1, 400):
        for split in range(1, MAX_PIECES + 1):
            assert tile_range(0, kv_pieces(n_tiles, split), n_tiles)[0] == 0


def test_narrow_block_table_never_cuts_and_long_prompts_take_wide_tiles():
    assert kv_split_of(32, 512, 1, (2 * MIN_PIECE_TILES * KV_TILE) // BLOCK - 1, 64) == 1
    assert kv_split_of(32, 512, 1, 4096, 64) == 768 // (32 * 9)
    assert q_tile_of(32, 15928, 16, 1962, 128) == 128      # the prefill workload of the benchmark
    assert q_tile_of(32, 512, 1, 512, 32) == 64            # a chunk without room for a prefix
    assert q_tile_of(32, 512, 1, 512, 4096) == 128         # the same chunk behind a wide table
    assert q_tile_of(32, 2048, 1, 2048, 128) == 64         # one prompt, too few wide tiles to hide its last one
    assert q_tile_of(32, 3072, 1, 3072, 192) == 128
    assert q_tile_of(32, 2560, 64, 40, 4096) == 64         # many short prompts
