"""Seeded synthetic inputs for the HetSeq training-step hot path.

This module only draws inputs (model shapes, initial parameters, sequence lengths,
token ids, masked-LM targets).  It holds none of the method's arithmetic and is the one
module that both the HIP path's callers and the CPU oracle's callers use, so that the
two sides see byte-identical inputs.  It imports neither of them.

The inputs stand in for the Wikipedia corpus the paper trains BERT on (section "BERT
Language Model"): same shapes and value distributions, no item of any dataset.
"""
from __future__ import annotations

import numpy as np

PAD_ID = 0
MASK_ID = 4
FIRST_REAL_ID = 5          # ids 0..4 are reserved (PAD = 0, MASK = 4)

# Model shapes.  Keys follow the C struct hs_model_cfg.
MODELS = {
    "tiny": dict(n_layers=1, hidden=128, n_heads=2, ffn=512, vocab=1000, max_pos=64, ln_eps=1e-12),
    "bert_base": dict(n_layers=12, hidden=768, n_heads=12, ffn=3072, vocab=30522, max_pos=512, ln_eps=1e-12),
    "bert_large": dict(n_layers=24, hidden=1024, n_heads=16, ffn=4096, vocab=30522, max_pos=512, ln_eps=1e-12),
}

# The five workloads, in the order they are numbered (0..4).
WORKLOADS = {
    0: dict(name="tiny_fp32", model="tiny", compute="fp32", ids="uniform", seed=1234,
            adam=dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-6)),
    1: dict(name="bert_base_L128_cap8192", model="bert_base", compute="bf16", ids="zipf", seed=1235,
            adam=dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8)),
    2: dict(name="bert_base_varlen_cap16384", model="bert_base", compute="bf16", ids="zipf", seed=1236,
            adam=dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8)),
    3: dict(name="bert_base_L256_hetero_8_24_56", model="bert_base", compute="bf16", ids="zipf", seed=1237,
            adam=dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8)),
    4: dict(name="bert_large_L512_4x32", model="bert_large", compute="bf16", ids="zipf", seed=1238,
            adam=dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8)),
}


def rng_for(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def init_params(layout, seed: int) -> np.ndarray:
    """float32 N(0, 0.02) for the whole flat buffer from one stream in layout order, then
    +1 on every LayerNorm gain (names ending in '.g').  `layout` is a list of
    (name, offset, rows, cols) from whichever side asks."""
    total = max(off + r * c for _, off, r, c in layout)
    theta = (rng_for(seed).standard_normal(total) * 0.02).astype(np.float32)
    for name, off, r, c in layout:
        if name.endswith(".g"):
            theta[off:off + r * c] += np.float32(1.0)
    return theta


def draw_ids(rng: np.random.Generator, n: int, vocab: int, dist: str) -> np.ndarray:
    """Token ids in [5, vocab): uniform, or Zipf with exponent 1.1 over ranks 1..vocab-5
    (id = 4 + rank) by inverse CDF on seeded uniforms."""
    if dist == "uniform":
        return rng.integers(FIRST_REAL_ID, vocab, size=n).astype(np.int32)
    if dist == "zipf":
        ranks = np.arange(1, vocab - FIRST_REAL_ID + 1, dtype=np.float64)
        cdf = np.cumsum(ranks ** -1.1)
        cdf /= cdf[-1]
        u = rng.random(n)
        r = np.searchsorted(cdf, u, side="left")
        r = np.minimum(r, len(ranks) - 1)
        return (FIRST_REAL_ID + r).astype(np.int32)
    raise ValueError(dist)


def n_targets(length: int) -> int:
    """Masked-LM targets of one sequence: 15% of its real tokens, at least one."""
    return max(1, int(np.floor(0.15 * length + 0.5)))


def make_micro_batch(rng: np.random.Generator, lens, L: int, vocab: int, dist: str) -> dict:
    """One padded micro-batch.  ids [B, L] int32 (PAD beyond each length, MASK at every
    target), lens [B] int32, mlm_pos [M] int32 = b * L + l ascending, mlm_label [M] int32
    (the original id at the target)."""
    lens = np.asarray(lens, dtype=np.int32)
    B = len(lens)
    assert np.all(lens >= 1) and np.all(lens <= L)
    ids = np.full((B, L), PAD_ID, dtype=np.int32)
    pos, lab = [], []
    for b in range(B):
        n = int(lens[b])
        ids[b, :n] = draw_ids(rng, n, vocab, dist)
        tgt = np.sort(rng.permutation(n)[:n_targets(n)])
        for l in tgt:
            pos.append(b * L + int(l))
            lab.append(int(ids[b, l]))
            ids[b, l] = MASK_ID
    return dict(ids=ids, lens=lens, mlm_pos=np.asarray(pos, dtype=np.int32),
                mlm_label=np.asarray(lab, dtype=np.int32), n_seq=B, n_real_tokens=int(lens.sum()))


def draw_lengths(rng: np.random.Generator, n: int, lo: int, hi: int) -> np.ndarray:
    """n sequence lengths uniform in [lo, hi]."""
    return rng.integers(lo, hi + 1, size=n).astype(np.int32)


def workload_micro_batches(idx: int) -> list:
    """The fixed-shape workloads (0, 1, 3, 4) as lists of micro-batches.  Workload 2 is
    built from draw_lengths + a batcher by its caller (batch formation is part of the
    method, not of input synthesis)."""
    wl = WORKLOADS[idx]
    vocab = MODELS[wl["model"]]["vocab"]
    rng = rng_for(wl["seed"])
    if idx == 0:
        return [make_micro_batch(rng, [16, 32, 48, 64], 64, vocab, wl["ids"])]
    if idx == 1:
        return [make_micro_batch(rng, [128] * 64, 128, vocab, wl["ids"])]
    if idx == 3:
        return [make_micro_batch(rng, [256] * b, 256, vocab, wl["ids"]) for b in (8, 24, 56)]
    if idx == 4:
        return [make_micro_batch(rng, [512] * 32, 512, vocab, wl["ids"]) for _ in range(4)]
    raise ValueError("workload 2 is formed by a batcher; see draw_lengths")


def concat_micro_batches(mbs: list) -> dict:
    """The single batch that holds every sequence of `mbs` (same padded length)."""
    L = mbs[0]["ids"].shape[1]
    assert all(mb["ids"].shape[1] == L for mb in mbs)
    ids = np.concatenate([mb["ids"] for mb in mbs], axis=0)
    lens = np.concatenate([mb["lens"] for mb in mbs])
    pos, lab, base = [], [], 0
    for mb in mbs:
        pos.append(mb["mlm_pos"].astype(np.int64) + base * L)
        lab.append(mb["mlm_label"])
        base += mb["ids"].shape[0]
    return dict(ids=ids, lens=lens, mlm_pos=np.concatenate(pos).astype(np.int32),
                mlm_label=np.concatenate(lab).astype(np.int32), n_seq=ids.shape[0],
                n_real_tokens=int(lens.sum()))


def step_micro_batches(seed: int, t: int, lens, L: int, vocab: int, dist: str, n_micro: int = 1, dropout: float = 0.0) -> list:
    """The micro-batches of update number t of a multi-step run: drawn from a generator seeded with
    seed + t, so that a run resumed after any number of updates sees the same data as an
    uninterrupted one (the seed is part of a checkpoint).  With dropout > 0 every micro-batch carries
    its dropout state: the run's seed and a stream number of its own (64 t + index)."""
    rng = rng_for(seed + t)
    out = [make_micro_batch(rng, lens, L, vocab, dist) for _ in range(n_micro)]
    if dropout > 0.0:
        for i, mb in enumerate(out):
            mb["drop"] = dict(p=dropout, seed=seed, stream=64 * t + i)
    return out


def mask_batch(rng: np.random.Generator, ids: np.ndarray, lens) -> dict:
    """Masked-LM targets for a padded batch whose tokens are given (for batches that come from a
    dataset): per sequence n_targets(len) distinct real positions get MASK, their ids become labels."""
    ids = np.array(ids, dtype=np.int32, copy=True)
    lens = np.asarray(lens, dtype=np.int32)
    B, L = ids.shape
    pos, lab = [], []
    for b in range(B):
        n = int(lens[b])
        for l in np.sort(rng.permutation(n)[:n_targets(n)]):
            pos.append(b * L + int(l))
            lab.append(int(ids[b, l]))
            ids[b, l] = MASK_ID
    return dict(ids=ids, lens=lens, mlm_pos=np.asarray(pos, dtype=np.int32), mlm_label=np.asarray(lab, dtype=np.int32),
                n_seq=B, n_real_tokens=int(lens.sum()))


# ---- translation workload (source / target pairs) ---------------------------------------------
EOS_ID = 2
S2S_MODELS = {
    "s2s_tiny": dict(n_enc=2, n_dec=2, hidden=128, n_heads=2, ffn=256, vocab=600, max_pos=64, ln_eps=1e-5),
    "transformer_base": dict(n_enc=6, n_dec=6, hidden=512, n_heads=8, ffn=2048, vocab=37000, max_pos=256, ln_eps=1e-5),
}


def make_pair_batch(rng: np.random.Generator, src_lens, tgt_lens, Ls: int, Lt: int, vocab: int, dist: str) -> dict:
    """One padded batch of sentence pairs.  src [B, Ls]; a target of length n is n - 1 drawn tokens followed
    by EOS: tgt_out [B, Lt] holds it, tgt_in [B, Lt] the same shifted right behind a leading EOS (the decoder's
    input).  PAD beyond the lengths."""
    src_lens = np.asarray(src_lens, dtype=np.int32)
    tgt_lens = np.asarray(tgt_lens, dtype=np.int32)
    B = len(src_lens)
    assert len(tgt_lens) == B and np.all(src_lens >= 1) and np.all(src_lens <= Ls) and np.all(tgt_lens >= 1) and np.all(tgt_lens <= Lt)
    src = np.full((B, Ls), PAD_ID, dtype=np.int32)
    tgt_in = np.full((B, Lt), PAD_ID, dtype=np.int32)
    tgt_out = np.full((B, Lt), PAD_ID, dtype=np.int32)
    for b in range(B):
        ns, nt = int(src_lens[b]), int(tgt_lens[b])
        src[b, :ns] = draw_ids(rng, ns, vocab, dist)
        y = np.concatenate([draw_ids(rng, nt - 1, vocab, dist), [EOS_ID]]).astype(np.int32)
        tgt_out[b, :nt] = y
        tgt_in[b, 0] = EOS_ID
        tgt_in[b, 1:nt] = y[:nt - 1]
    return dict(src=src, src_lens=src_lens, tgt_in=tgt_in, tgt_out=tgt_out, tgt_lens=tgt_lens, n_seq=B,
                n_src_tokens=int(src_lens.sum()), n_tgt_tokens=int(tgt_lens.sum()))


def draw_pair_lengths(rng: np.random.Generator, n: int, lo: int, hi: int):
    """Source lengths uniform in [lo, hi]; each target length is its source length times a factor uniform
    in [0.8, 1.25], clipped to [lo, hi] (sentence pairs of similar length, as translation corpora have)."""
    s = rng.integers(lo, hi + 1, size=n)
    t = np.clip(np.rint(s * rng.uniform(0.8, 1.25, size=n)), lo, hi).astype(np.int32)
    return s.astype(np.int32), t


def pair_workload(seed=1240, B=128, L=32):
    """The translation workload's batch: 128 sentence pairs in buffers of 32 positions per side (4096 positions per
    side, the per-worker max-tokens of table 1), lengths uniform in [16, 32] with targets 0.8 .. 1.25 times the source."""
    rng = rng_for(seed)
    sl, tl = draw_pair_lengths(rng, B, L // 2, L)
    return make_pair_batch(rng, sl, tl, L, L, S2S_MODELS["transformer_base"]["vocab"], "zipf")
