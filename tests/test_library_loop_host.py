"""Host-side entry points of the multi-step loop: learning-rate schedule and checkpoint files
(no GPU; the library is loaded, no kernel is launched)."""
import os

import numpy as np
import pytest

from oracle import hetseq_oracle as O
from paper_2009_14783_amd import binding as hs
from paper_2009_14783_amd import synth


def test_lr_linear_matches_oracle_and_rejects_bad_arguments():
    for max_lr, warmup, total in ((1e-4, 10000, 1000000), (3e-4, 7, 40), (1.0, 0, 10), (2e-3, 5, 5)):
        for t in sorted({1, 2, max(1, warmup - 1), max(1, warmup), warmup + 1, (warmup + total) // 2 + 1, total - 1 or 1, total, total + 3}):
            assert hs.hs_lr_linear(t, max_lr, warmup, total) == O.lr_linear(t, max_lr, warmup, total), (t, warmup, total)
    for bad in ((0, 1e-4, 2, 10), (1, 1e-4, -1, 10), (1, 1e-4, 11, 10), (1, -1.0, 2, 10), (1, float("nan"), 2, 10), (1, 1e-4, 0, 0)):
        with pytest.raises(hs.HsError):
            hs.hs_lr_linear(*bad)


def _header(cfg, n, step=17):
    h = hs.hs_ckpt_header()
    h.cfg = cfg
    h.n_params, h.epoch, h.step, h.seed = n, 2, step, 1234567890123
    h.max_lr, h.warmup, h.total = 1e-4, 10000, 1000000
    h.beta1, h.beta2, h.eps, h.weight_decay = 0.9, 0.999, 1e-8, 0.01
    return h


def test_checkpoint_round_trip_is_bit_exact(tmp_path):
    cfg = hs.make_cfg(**synth.MODELS["tiny"], compute=hs.HS_FP32)
    n = hs.hs_param_count(cfg)
    rng = np.random.default_rng(5)
    w, m, v = (rng.standard_normal(n).astype(np.float32) for _ in range(3))
    w[:4] = [np.float32("nan"), np.float32("inf"), -0.0, np.float32(1e-42)]      # bit patterns, not values
    path = str(tmp_path / "state.hsckpt")
    hs.hs_checkpoint_write(path, _header(cfg, n), w, m, v)
    assert not os.path.exists(path + ".tmp")
    head = hs.hs_checkpoint_read_header(path)
    assert (head.n_params, head.epoch, head.step, head.seed) == (n, 2, 17, 1234567890123)
    assert (head.max_lr, head.warmup, head.total) == (1e-4, 10000, 1000000)
    assert (head.beta1, head.beta2, head.eps, head.weight_decay) == (0.9, 0.999, 1e-8, 0.01)
    assert head.cfg.hidden == cfg.hidden and head.cfg.vocab == cfg.vocab
    w2, m2, v2 = (np.empty(n, dtype=np.float32) for _ in range(3))
    hs.hs_checkpoint_read(path, w2, m2, v2)
    for a, b in ((w, w2), (m, m2), (v, v2)):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    assert os.path.getsize(path) == 8 + 120 + 12 * n + 8


def test_checkpoint_errors(tmp_path):
    cfg = hs.make_cfg(**synth.MODELS["tiny"], compute=hs.HS_FP32)
    n = hs.hs_param_count(cfg)
    z = np.zeros(n, dtype=np.float32)
    path = str(tmp_path / "state.hsckpt")
    with pytest.raises(hs.HsError):                      # wrong parameter count for the model
        hs.hs_checkpoint_write(path, _header(cfg, n - 1), z[:-1].copy(), z[:-1].copy(), z[:-1].copy())
    with pytest.raises(hs.HsError):                      # directory does not exist
        hs.hs_checkpoint_write(str(tmp_path / "no" / "dir" / "x"), _header(cfg, n), z, z, z)
    with pytest.raises(hs.HsError):                      # no such file
        hs.hs_checkpoint_read_header(path)
    hs.hs_checkpoint_write(path, _header(cfg, n), z, z, z)
    blob = bytearray(open(path, "rb").read())
    short = np.zeros(n - 1, dtype=np.float32)
    with pytest.raises(hs.HsError):                      # caller's arrays of another size
        hs.hs_checkpoint_read(path, short, short.copy(), short.copy())
    bad = str(tmp_path / "flipped")
    flipped = bytearray(blob); flipped[len(blob) // 2] ^= 0x40
    open(bad, "wb").write(flipped)
    with pytest.raises(hs.HsError, match="checksum"):
        hs.hs_checkpoint_read(bad, z.copy(), z.copy(), z.copy())
    open(bad, "wb").write(blob[: len(blob) - 100])
    with pytest.raises(hs.HsError, match="truncated|checksum"):
        hs.hs_checkpoint_read(bad, z.copy(), z.copy(), z.copy())
    open(bad, "wb").write(b"NOTACKPT" + blob[8:])
    with pytest.raises(hs.HsError, match="magic"):
        hs.hs_checkpoint_read_header(bad)
