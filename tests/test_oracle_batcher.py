"""Pins of the batch-formation oracle: brute-force properties and the degenerate cases
whose answers the workload descriptions print (CPU only)."""
import numpy as np
import pytest

from oracle import batcher as OB
from paper_2009_14783_amd import synth


def check_batches(lengths, bw, cap, mode, seq_index, offsets, pad_lens):
    n = len(lengths)
    assert sorted(seq_index) == list(range(n))                     # every index exactly once
    assert offsets[0] == 0 and offsets[-1] == n and len(offsets) == len(pad_lens) + 1
    for j, pad in enumerate(pad_lens):
        members = seq_index[offsets[j]:offsets[j + 1]]
        assert len(members) >= 1
        lens = [int(lengths[i]) for i in members]
        assert all(pad - bw < ln <= pad for ln in lens) and pad % bw == 0
        used = sum(lens) if mode == 0 else len(lens) * pad
        assert used <= cap
    # order: (length, index) ascending across the whole output
    keys = [(int(lengths[i]), i) for i in seq_index]
    assert keys == sorted(keys)


@pytest.mark.parametrize("mode", [0, 1])
def test_properties_on_random_lengths(mode):
    rng = synth.rng_for(2)
    lengths = synth.draw_lengths(rng, 500, 64, 512)
    si, off, pl = OB.make_batches(lengths, 64, 16384, mode)
    check_batches(lengths, 64, 16384, mode, si, off, pl)
    # greedy maximality: a batch that is followed by another batch of the same bucket could
    # not have taken that batch's first sequence
    for j in range(len(pl) - 1):
        if pl[j] == pl[j + 1]:
            nxt = int(lengths[si[off[j + 1]]])
            members = si[off[j]:off[j + 1]]
            used = sum(int(lengths[i]) for i in members) + nxt if mode == 0 else (len(members) + 1) * pl[j]
            assert used > 16384


def test_degenerate_full_length_batches():
    # seq len 128 under a cap of 8192 tokens -> 64 sequences; 512 under 16384 -> 32
    si, off, pl = OB.make_batches([128] * 64, 64, 8192, 0)
    assert off == [0, 64] and pl == [128] and si == list(range(64))
    si, off, pl = OB.make_batches([512] * 96, 64, 16384, 0)
    assert off == [0, 32, 64, 96] and pl == [512] * 3
    si, off, pl = OB.make_batches([512] * 96, 64, 16384, 1)
    assert off == [0, 32, 64, 96]


def test_hand_worked_small_case():
    # lengths:        idx0  1  2  3  4  5  6
    lengths = [5, 3, 9, 4, 8, 3, 12]
    # sorted by (len, idx): 1(3) 5(3) 3(4) 0(5) 4(8) 2(9) 6(12); bucket width 4 -> pads 4 4 4 8 8 12 12
    # cap 7 real tokens: [1,5] (6; +4 > 7) | [3] (bucket ends) | [0] (5; +8 > 7) | [4] | [2] | [6]
    si, off, pl = OB.make_batches(lengths, 4, 12, 0)
    # cap 12: bucket 4: 3+3+4 = 10 -> [1,5,3]; bucket 8: 5 then 5+8 = 13 > 12 -> [0] | [4]; bucket 12: [2] | [6]
    assert si == [1, 5, 3, 0, 4, 2, 6]
    assert off == [0, 3, 4, 5, 6, 7]
    assert pl == [4, 8, 8, 12, 12]
    # padded-size cap 16: bucket 4 (pad 4): 3 seqs = 12 <= 16 -> [1,5,3]; bucket 8: 2 x 8 = 16 -> [0,4];
    # bucket 12: 2 x 12 = 24 > 16 -> [2] | [6]
    si, off, pl = OB.make_batches(lengths, 4, 16, 1)
    assert si == [1, 5, 3, 0, 4, 2, 6] and off == [0, 3, 5, 6, 7] and pl == [4, 8, 12, 12]


def test_empty_and_single():
    assert OB.make_batches([], 64, 100, 0) == ([], [0], [])
    assert OB.make_batches([7], 64, 100, 0) == ([0], [0, 1], [64])
