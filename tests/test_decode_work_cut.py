"""The index arithmetic of the decode-attention work cut, restated on the host.

The attention kernels cut all (sequence, head group, block) units into equal
contiguous ranges, one per worker, and leave one partial state per piece in
row `(worker + sequence * Hg + head_group) * Gs + head_in_group`; the merge
kernel finds the pieces of a head from `worker_of(first unit) .. worker_of(last unit)`.
These tests check the properties that make that scheme sound, for random
batches: every unit has exactly one owner, pieces never share a row, every row
is inside the buffer, and the merge kernel's worker range is exactly the set of
workers that hold a piece of the head.  (Pure host arithmetic; the kernels are
checked against the oracle in the GPU tests.)
"""
import numpy as np
import pytest


def worker_begin(w, U, W):
    return w * U // W


def worker_of(u, U, W):
    return ((u + 1) * W + U - 1) // U - 1


def pieces(ctx, Hkv, Gs, n_workers):
    """(worker, seq, head group, first block, blocks) for every piece, as the attention kernels walk them."""
    nb = (ctx + 1 + 15) // 16
    prefix = np.concatenate([[0], np.cumsum(nb)])
    Hg = Hkv // Gs
    U = int(prefix[-1]) * Hg
    W = min(n_workers // Gs, U, max(8 * len(ctx) * Hg, U // 16))   # few sequences: at most eight workers per head group, or 16 blocks each
    out = []
    for w in range(W):
        u, u_end = worker_begin(w, U, W), worker_begin(w + 1, U, W)
        assert u < u_end, "no empty ranges when W <= U"
        seq = int(np.searchsorted(prefix * Hg, u, side="right") - 1)
        while u < u_end:
            while prefix[seq + 1] * Hg <= u:
                seq += 1
            r = u - prefix[seq] * Hg
            hg, blk0 = divmod(int(r), int(nb[seq]))
            n = min(int(nb[seq]) - blk0, u_end - u)
            out.append((w, seq, hg, blk0, n))
            u += n
    return out, prefix, U, W, Hg


@pytest.mark.parametrize("seed", range(12))
def test_cut_covers_every_block_once_and_rows_are_unique(seed):
    rng = np.random.default_rng(seed)
    B = int(rng.integers(1, 40))
    Gs = int(rng.choice([1, 2, 4]))
    Hkv = Gs * int(rng.integers(1, 9))
    n_workers = 4 * int(rng.integers(1, 65))
    ctx = rng.integers(0, 700, size=B)
    ps, prefix, U, W, Hg = pieces(ctx, Hkv, Gs, n_workers)
    nb = np.diff(prefix)
    # every (sequence, head group, block) exactly once
    seen = np.zeros((B, Hg, int(nb.max())), dtype=np.int32)
    for w, seq, hg, blk0, n in ps:
        seen[seq, hg, blk0:blk0 + n] += 1
    for s in range(B):
        assert (seen[s, :, :nb[s]] == 1).all() and (seen[s, :, nb[s]:] == 0).all()
    # ranges are balanced: they differ by at most one unit
    sizes = [worker_begin(w + 1, U, W) - worker_begin(w, U, W) for w in range(W)]
    assert max(sizes) - min(sizes) <= 1
    # one row per piece and head of the group, inside the buffer of n_workers + B * Hkv rows
    rows = set()
    for w, seq, hg, _, _ in ps:
        for hi in range(Gs):
            row = (w + seq * Hg + hg) * Gs + hi
            assert 0 <= row < n_workers + B * Hkv
            assert row not in rows
            rows.add(row)


@pytest.mark.parametrize("seed", range(12))
def test_merge_kernel_finds_exactly_the_workers_that_hold_a_piece(seed):
    rng = np.random.default_rng(100 + seed)
    B = int(rng.integers(1, 30))
    Gs = int(rng.choice([1, 2, 4]))
    Hkv = Gs * int(rng.integers(1, 6))
    n_workers = 4 * int(rng.integers(1, 40))
    ctx = rng.integers(0, 1500, size=B)
    ps, prefix, U, W, Hg = pieces(ctx, Hkv, Gs, n_workers)
    holders = {}
    for w, seq, hg, _, _ in ps:
        holders.setdefault((seq, hg), []).append(w)
    for seq in range(B):
        nb = int(prefix[seq + 1] - prefix[seq])
        for hg in range(Hg):
            u0 = int(prefix[seq]) * Hg + hg * nb
            w_first, w_last = worker_of(u0, U, W), worker_of(u0 + nb - 1, U, W)
            assert holders[(seq, hg)] == list(range(w_first, w_last + 1))


def test_worker_of_inverts_worker_begin():
    for U, W in [(1, 1), (7, 3), (100, 100), (1000, 64), (18480, 512), (5, 5), (4097, 2048)]:
        W = min(W, U)
        for w in range(W):
            lo, hi = worker_begin(w, U, W), worker_begin(w + 1, U, W)
            assert worker_of(lo, U, W) == w and worker_of(hi - 1, U, W) == w
