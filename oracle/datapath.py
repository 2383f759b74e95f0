"""Plain Python model of the host data path (TEST INFRASTRUCTURE ONLY; never used by the product).

What the paper fixes (HetSeq, "Distributed GPU Training on Heterogeneous Infrastructure"):
* Section "Dataset and Dataloader": the dataset is split into shards; the lengths of the files are
  accumulated and the index of a training instance is mapped to an offset inside its shard; shuffling
  must be reproducible.
* Section "Forward Pass": batches are formed under a max-instances or max-tokens criterion
  (`oracle.batcher.make_batches`).
* Section "Checkpointing" (seed handling): the order of an epoch is a function of the seed and the
  epoch number.
* Section "Prefetch and Cache": the next batches are fetched while the current one trains, and a
  least-recently-used cache keeps instances in memory.

Readings where the paper is silent: the batches of an epoch are formed once over all lengths, their
order is shuffled by Fisher-Yates driven by the Philox generator (for i = n-1 .. 1: swap i with
word 0 of block (i, epoch, tag) modulo i+1), and worker `rank` of `world` takes the shuffled batches
rank, rank + world, ...  Shard file: the 8 bytes "HSSHARD1", int64 n_seq, int64 n_tokens, int32
lengths[n_seq], int32 tokens[n_tokens] (little-endian).

Pins (tests/test_oracle_datapath.py): index map against brute force, the shuffle is a permutation
that depends on seed and epoch only and deals every batch to exactly one worker, the LRU model
against a hand-worked trace.
"""
from __future__ import annotations

import struct
from collections import OrderedDict

import numpy as np

from . import batcher
from .hetseq_oracle import philox4x32_10

SHUFFLE_TAG = 0x5AFF1E


def write_shard(path: str, sequences: list):
    lengths = np.array([len(s) for s in sequences], dtype=np.int32)
    tokens = np.concatenate([np.asarray(s, dtype=np.int32) for s in sequences]) if sequences else np.zeros(0, np.int32)
    with open(path, "wb") as f:
        f.write(b"HSSHARD1")
        f.write(struct.pack("<qq", len(sequences), tokens.size))
        f.write(lengths.tobytes())
        f.write(tokens.tobytes())


def read_shard(path: str):
    with open(path, "rb") as f:
        assert f.read(8) == b"HSSHARD1"
        n_seq, n_tok = struct.unpack("<qq", f.read(16))
        lengths = np.frombuffer(f.read(4 * n_seq), dtype=np.int32)
        tokens = np.frombuffer(f.read(4 * n_tok), dtype=np.int32)
    return lengths, tokens


def index_map(shard_sizes, i: int):
    """Global instance i -> (shard, row inside the shard): shards are concatenated in order."""
    acc = 0
    for s, n in enumerate(shard_sizes):
        if i < acc + n:
            return s, i - acc
        acc += n
    raise IndexError(i)


def shuffle_order(n: int, seed: int, epoch: int) -> np.ndarray:
    """Permutation of range(n) for one epoch."""
    order = np.arange(n, dtype=np.int64)
    if n < 2:
        return order
    idx = np.arange(n, dtype=np.uint64)
    ctr = np.empty((n, 4), dtype=np.uint32)
    ctr[:, 0] = (idx & np.uint64(0xFFFFFFFF)).astype(np.uint32)
    ctr[:, 1] = (idx >> np.uint64(32)).astype(np.uint32)
    ctr[:, 2] = np.uint32(epoch & 0xFFFFFFFF)
    ctr[:, 3] = np.uint32(SHUFFLE_TAG)
    words = philox4x32_10(ctr, (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF))[:, 0]
    for i in range(n - 1, 0, -1):
        j = int(words[i]) % (i + 1)
        order[i], order[j] = order[j], order[i]
    return order


def epoch_batches(lengths, bucket_width, max_tokens, cap_mode, seed, epoch, world=1, rank=0):
    """The batches (pad_len, [instance indices]) that worker `rank` sees in this epoch, in order."""
    seq_index, offsets, pads = batcher.make_batches(lengths, bucket_width, max_tokens, cap_mode)
    n = len(pads)
    order = shuffle_order(n, seed, epoch)
    mine = order[rank::world]
    return [(int(pads[b]), [int(x) for x in seq_index[offsets[b]:offsets[b + 1]]]) for b in mine]


class LruModel:
    """Least-recently-used cache over instance indices, `capacity` instances; counts hits and loads."""

    def __init__(self, capacity: int):
        self.capacity, self.d, self.hits, self.loads = capacity, OrderedDict(), 0, 0

    def touch(self, i: int):
        if self.capacity > 0 and i in self.d:
            self.d.move_to_end(i)
            self.hits += 1
            return
        self.loads += 1
        if self.capacity > 0:
            self.d[i] = True
            if len(self.d) > self.capacity:
                self.d.popitem(last=False)
