"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, its parameter layout and batch former agree with the oracle's, and bad
arguments come back as error codes."""
import os
import re

import numpy as np
import pytest

from oracle import batcher as OB
from oracle import hetseq_oracle as O
from paper_2009_14783_amd import binding as hs
from paper_2009_14783_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "hetseq_hip.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(hs_[a-z0-9_]+)\s*\(", header))
    assert {"hs_encoder_fwd", "hs_encoder_bwd", "hs_mlm_loss", "hs_grad_accum_normalize", "hs_adam_step",
            "hs_make_batches"} <= declared
    lib = hs.lib()
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert declared == set(hs.EXPORTS)                   # the binding carries the same names


@pytest.mark.parametrize("model", ["tiny", "bert_base", "bert_large"])
def test_layout_matches_oracle_layout(model):
    m = synth.MODELS[model]
    cfg = hs.make_cfg(**m)
    assert hs.hs_param_layout(cfg) == O.param_layout(O.ModelCfg(**m))
    assert hs.hs_param_count(cfg) == O.param_count(O.ModelCfg(**m))
    for _, off, r, c in hs.hs_param_layout(cfg):
        if r > 1:
            assert off % 8 == 0                            # 16-byte aligned rows in bf16


def test_sizes_and_invalid_configs():
    cfg = hs.make_cfg(**synth.MODELS["bert_base"])
    assert hs.hs_acts_bytes(cfg, 64, 128, 1216) > 64 * 128 * 768 * 2 * 12
    assert hs.hs_workspace_bytes(cfg, 64, 128, 1216) >= 1216 * 30528 * 4
    assert hs.hs_workspace_bytes(cfg, 64, 128, 0) > 0
    bad = hs.make_cfg(n_layers=1, hidden=100, n_heads=2, ffn=512, vocab=1000, max_pos=64)
    assert hs.hs_param_count(bad) == 0
    with pytest.raises(hs.HsError) as e:
        hs.hs_ctx_create(bad)
    assert e.value.status == 2 and "hidden" in str(e.value)
    ctx = hs.hs_ctx_create(cfg)
    hs.hs_ctx_destroy(ctx)


@pytest.mark.parametrize("model", ["s2s_tiny", "transformer_base"])
def test_pair_model_layout_matches_oracle_layout(model):
    from oracle import seq2seq_oracle as S
    m = synth.S2S_MODELS[model]
    cfg = hs.make_s2s_cfg(**m)
    assert hs.hs_s2s_param_layout(cfg) == S.param_layout(S.S2SCfg(**m))
    assert hs.hs_s2s_param_count(cfg) == S.param_count(S.S2SCfg(**m))
    for _, off, r, c in hs.hs_s2s_param_layout(cfg):
        if r > 1:
            assert off % 8 == 0                            # 16-byte aligned rows in bf16


def test_pair_model_sizes_and_invalid_configs():
    cfg = hs.make_s2s_cfg(**synth.S2S_MODELS["transformer_base"])
    small, big = hs.hs_s2s_acts_bytes(cfg, 16, 32, 32), hs.hs_s2s_acts_bytes(cfg, 128, 32, 32)
    assert 0 < small < big and hs.hs_s2s_acts_bytes(cfg, 128, 64, 32) > big
    assert hs.hs_s2s_workspace_bytes(cfg, 128, 32, 32) >= 128 * 32 * 37056 * 6      # fp32 logits and their bf16 gradient
    bad = hs.make_s2s_cfg(n_enc=1, n_dec=0, hidden=128, n_heads=2, ffn=256, vocab=100, max_pos=64)
    assert hs.hs_s2s_param_count(bad) == 0
    with pytest.raises(hs.HsError) as e:
        hs.hs_s2s_ctx_create(bad)
    assert e.value.status == 2 and "n_dec" in str(e.value)
    bad = hs.make_s2s_cfg(n_enc=1, n_dec=1, hidden=128, n_heads=4, ffn=256, vocab=100, max_pos=64)
    with pytest.raises(hs.HsError):
        hs.hs_s2s_ctx_create(bad)                          # hidden / n_heads must be 64
    ctx = hs.hs_s2s_ctx_create(cfg)
    hs.hs_ctx_destroy(ctx)


@pytest.mark.parametrize("mode", [0, 1])
def test_batcher_bit_exact_against_oracle(mode):
    rng = synth.rng_for(1236)
    lengths = synth.draw_lengths(rng, 4096, 64, 512)                 # the variable-length workload
    seq, offs, pads = hs.hs_make_batches(lengths, 64, 16384, mode)
    oseq, ooffs, opads = OB.make_batches(lengths, 64, 16384, mode)
    assert seq.tolist() == oseq and offs.tolist() == ooffs and pads.tolist() == opads
    for bw, cap in [(1, 50), (8, 64), (64, 8192), (7, 1000)]:
        lengths = synth.draw_lengths(synth.rng_for(bw * 1000 + cap), 777, 1, min(cap, 50))
        seq, offs, pads = hs.hs_make_batches(lengths, bw, cap, mode)
        oseq, ooffs, opads = OB.make_batches(lengths, bw, cap, mode)
        assert seq.tolist() == oseq and offs.tolist() == ooffs and pads.tolist() == opads


def test_batcher_degenerate_and_errors():
    seq, offs, pads = hs.hs_make_batches([128] * 64, 64, 8192, 0)
    assert offs.tolist() == [0, 64] and pads.tolist() == [128]
    seq, offs, pads = hs.hs_make_batches([512] * 96, 64, 16384, 0)
    assert offs.tolist() == [0, 32, 64, 96]
    seq, offs, pads = hs.hs_make_batches([], 64, 100, 0)
    assert seq.size == 0 and offs.tolist() == [0] and pads.size == 0
    with pytest.raises(hs.HsError):
        hs.hs_make_batches([10, 200], 64, 100, 0)                     # 200 real tokens cannot fit a cap of 100
    with pytest.raises(hs.HsError):
        hs.hs_make_batches([10, 0], 64, 100, 0)
    with pytest.raises(hs.HsError):
        hs.hs_make_batches([10], 0, 100, 0)
