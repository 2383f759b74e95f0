"""Plain-Python oracle of batch formation under a max-tokens cap (test infrastructure only).

The paper (section "Forward Pass") forms batches that satisfy a criterion such as a
maximum number of instances or a maximum number of tokens, and allows the last batch
to be partially filled (section "Optimizer and Learning Rate Scheduler").  The paper
does not say more, so the reading taken here is:

* sequences are ordered by (length, original index) - a stable sort, which makes the
  result unique;
* a sequence of length n belongs to the bucket whose padded length is
  ceil(n / bucket_width) * bucket_width;
* inside a bucket, in sorted order, a sequence joins the open batch unless that would
  break the cap, in which case the open batch is emitted and a new one starts;
  cap_mode 0 caps the number of REAL tokens (sum of lengths), cap_mode 1 caps the
  padded size (sequences x padded length);
* the last batch of a bucket may be partial; batches come out bucket by bucket.

This module shares nothing with the C++ batcher of the HIP library.
"""
from __future__ import annotations


def make_batches(lengths, bucket_width: int, max_tokens: int, cap_mode: int = 0):
    """Returns (seq_index, batch_offsets, batch_pad_len): batch j holds the sequences
    seq_index[batch_offsets[j]:batch_offsets[j+1]], padded to batch_pad_len[j]."""
    assert bucket_width >= 1 and max_tokens >= 1 and cap_mode in (0, 1)
    n = len(lengths)
    order = sorted(range(n), key=lambda i: (int(lengths[i]), i))
    seq_index, offsets, pad_lens = [], [0], []
    open_count, open_tokens, open_pad = 0, 0, None
    for i in order:
        ln = int(lengths[i])
        assert ln >= 1
        pad = -(-ln // bucket_width) * bucket_width
        cost = ln if cap_mode == 0 else pad
        assert cost <= max_tokens, "a single sequence exceeds the cap"
        if open_count > 0:
            would = open_tokens + ln if cap_mode == 0 else (open_count + 1) * pad
            if pad != open_pad or would > max_tokens:
                offsets.append(len(seq_index))
                pad_lens.append(open_pad)
                open_count, open_tokens = 0, 0
        seq_index.append(i)
        open_count += 1
        open_tokens += ln
        open_pad = pad
    if open_count > 0:
        offsets.append(len(seq_index))
        pad_lens.append(open_pad)
    return seq_index, offsets, pad_lens
