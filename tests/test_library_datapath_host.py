"""The native host data path against the oracle's model (no GPU): index map, batches, shuffle, dealing to
workers, batch contents, cache statistics, error handling."""
import os

import numpy as np
import pytest

from oracle import datapath as D
from paper_2009_14783_amd import binding as hs


def make_shards(tmp_path, rng, sizes, lo=1, hi=200, writer="oracle"):
    paths, seqs = [], []
    for s, n in enumerate(sizes):
        shard = [rng.integers(5, 30000, size=int(rng.integers(lo, hi + 1))).astype(np.int32) for _ in range(n)]
        p = str(tmp_path / f"part{s:03d}.shard")
        if writer == "oracle":
            D.write_shard(p, shard)
        else:
            hs.hs_shard_write(p, shard)
        paths.append(p)
        seqs += shard
    return paths, seqs


def test_both_shard_writers_give_the_same_bytes(tmp_path):
    rng = np.random.default_rng(3)
    a, _ = make_shards(tmp_path / "a", rng, [4, 0, 3]) if (tmp_path / "a").mkdir() is None else None
    rng = np.random.default_rng(3)
    b, _ = make_shards(tmp_path / "b", rng, [4, 0, 3], writer="native") if (tmp_path / "b").mkdir() is None else None
    for pa, pb in zip(a, b):
        assert open(pa, "rb").read() == open(pb, "rb").read()


def test_index_map_and_lengths(tmp_path):
    rng = np.random.default_rng(1)
    sizes = [7, 1, 0, 12, 5]
    paths, seqs = make_shards(tmp_path, rng, sizes)
    ds = hs.Dataset(paths)
    assert len(ds) == sum(sizes)
    assert ds.lengths().tolist() == [len(q) for q in seqs]
    for i in range(len(ds)):
        assert ds.locate(i) == D.index_map(sizes, i)
    with pytest.raises(hs.HsError):
        ds.locate(len(ds))
    ds.close()


@pytest.mark.parametrize("world,cache,prefetch", [(1, 0, 1), (1, 64, 3), (3, 1000, 2)])
def test_epochs_match_the_model(tmp_path, world, cache, prefetch):
    rng = np.random.default_rng(5)
    paths, seqs = make_shards(tmp_path, rng, [120, 80, 200, 33], lo=1, hi=300)
    lengths = np.array([len(q) for q in seqs], dtype=np.int32)
    for rank in range(world):
        ds = hs.Dataset(paths, cache_instances=cache, prefetch_batches=prefetch)
        model = D.LruModel(cache)
        for epoch in (0, 1, 2):
            want = D.epoch_batches(lengths, 64, 4096, 0, seed=99, epoch=epoch, world=world, rank=rank)
            n = ds.begin_epoch(99, epoch, 64, 4096, 0, world, rank)
            assert n == len(want)
            for pad, idx in want:
                assert ds.peek() == (len(idx), pad)
                ids, lens, inst = ds.next()
                assert inst.tolist() == idx and lens.tolist() == [len(seqs[i]) for i in idx]
                for r, i in enumerate(idx):
                    assert np.array_equal(ids[r, :lens[r]], seqs[i]) and not ids[r, lens[r]:].any()
                    model.touch(i)
            assert ds.peek() == (0, 0)
            with pytest.raises(StopIteration):
                ds.next()
            junk = np.zeros(4, np.int32)
            assert hs.lib().hs_dataset_next(ds.h, junk.ctypes.data, junk.ctypes.data, None) == 4      # HS_ERR_STATE: the epoch is over
            assert ds.stats() == (model.loads, model.hits)
        if cache >= len(seqs):
            assert model.hits > 0          # second and third epoch are served from memory
        ds.close()


def test_abandoning_an_epoch_and_restarting_it(tmp_path):
    rng = np.random.default_rng(8)
    paths, seqs = make_shards(tmp_path, rng, [50, 50])
    lengths = np.array([len(q) for q in seqs], dtype=np.int32)
    ds = hs.Dataset(paths, cache_instances=0, prefetch_batches=4)
    n = ds.begin_epoch(1, 0, 64, 1024)
    ds.next()
    n2 = ds.begin_epoch(1, 0, 64, 1024)            # worker thread of the first attempt is stopped and replaced
    assert n2 == n
    want = D.epoch_batches(lengths, 64, 1024, 0, seed=1, epoch=0)
    for pad, idx in want:
        _, _, inst = ds.next()
        assert inst.tolist() == idx
    ds.close()                                     # closing with nothing left to do
    ds = hs.Dataset(paths, prefetch_batches=2)
    ds.begin_epoch(1, 0, 64, 1024)
    ds.close()                                     # closing in the middle of an epoch


def test_errors(tmp_path):
    with pytest.raises(hs.HsError):
        hs.Dataset([str(tmp_path / "missing.shard")])
    bad = str(tmp_path / "bad.shard")
    open(bad, "wb").write(b"NOTSHARD" + bytes(16))
    with pytest.raises(hs.HsError):
        hs.Dataset([bad])
    rng = np.random.default_rng(2)
    paths, _ = make_shards(tmp_path, rng, [5])
    blob = open(paths[0], "rb").read()
    open(bad, "wb").write(blob[:-4])
    with pytest.raises(hs.HsError, match="truncated"):
        hs.Dataset([bad])
    ds = hs.Dataset(paths)
    with pytest.raises(hs.HsError):
        ds.begin_epoch(0, 0, 64, 16)               # a sequence longer than the cap cannot be batched
    with pytest.raises(hs.HsError):
        ds.begin_epoch(0, 0, 64, 4096, 0, 2, 2)    # rank outside the world
    ds.close()
    with pytest.raises(hs.HsError):
        hs.Dataset(paths, prefetch_batches=0)
