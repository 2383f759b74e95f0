"""Pins of the oracle's data-path model (CPU only)."""
import numpy as np

from oracle import datapath as D


def test_index_map_against_brute_force():
    sizes = [3, 0, 5, 1]
    flat = [(s, r) for s, n in enumerate(sizes) for r in range(n)]
    for i, want in enumerate(flat):
        assert D.index_map(sizes, i) == want


def test_shard_round_trip(tmp_path):
    seqs = [[5, 6, 7], [9], list(range(10, 30))]
    p = str(tmp_path / "a.shard")
    D.write_shard(p, seqs)
    lengths, tokens = D.read_shard(p)
    assert lengths.tolist() == [3, 1, 20] and tokens.tolist() == sum(seqs, [])


def test_shuffle_is_a_reproducible_permutation():
    for n in (0, 1, 2, 17, 1000):
        a = D.shuffle_order(n, 42, 3)
        assert sorted(a.tolist()) == list(range(n))
        assert np.array_equal(a, D.shuffle_order(n, 42, 3))
    a, b, c = D.shuffle_order(1000, 42, 3), D.shuffle_order(1000, 42, 4), D.shuffle_order(1000, 43, 3)
    assert not np.array_equal(a, b) and not np.array_equal(a, c)
    # every position is hit about equally often as the landing place of element 0 (coarse uniformity check)
    where = np.array([int(np.where(D.shuffle_order(8, s, 0) == 0)[0][0]) for s in range(4000)])
    counts = np.bincount(where, minlength=8)
    assert counts.min() > 400 and counts.max() < 600


def test_every_batch_goes_to_exactly_one_worker():
    rng = np.random.default_rng(1)
    lengths = rng.integers(1, 200, size=500).astype(np.int32)
    whole = D.epoch_batches(lengths, 64, 2048, 0, seed=7, epoch=2)
    parts = [D.epoch_batches(lengths, 64, 2048, 0, seed=7, epoch=2, world=3, rank=r) for r in range(3)]
    assert sum(len(p) for p in parts) == len(whole)
    dealt = [None] * len(whole)
    for r, p in enumerate(parts):
        for k, b in enumerate(p):
            dealt[r + 3 * k] = b
    assert dealt == whole
    seen = sorted(i for _, idx in whole for i in idx)
    assert seen == list(range(500))
    for pad, idx in whole:
        assert all(lengths[i] <= pad for i in idx) and sum(int(lengths[i]) for i in idx) <= 2048


def test_lru_model_hand_worked_trace():
    c = D.LruModel(2)
    for i in (1, 2, 1, 3, 2, 1):     # 1 miss, 2 miss, 1 hit, 3 miss (evicts 2), 2 miss (evicts 1), 1 miss (evicts 3)
        c.touch(i)
    assert (c.hits, c.loads) == (1, 5)
    z = D.LruModel(0)
    for i in (1, 1, 1):
        z.touch(i)
    assert (z.hits, z.loads) == (0, 3)
