"""Pins of the translation-workload oracle (oracle/seq2seq_oracle.py) against what the mathematics and the
cited definitions fix.  CPU only."""
import math

import numpy as np
import pytest
from scipy.special import logsumexp

from oracle import seq2seq_oracle as S
from paper_2009_14783_amd import synth

CFG = S.S2SCfg(n_enc=1, n_dec=2, hidden=16, n_heads=2, ffn=24, vocab=31, max_pos=16)


def _theta(cfg, seed, dtype=np.float64, spread=0.3):
    rng = np.random.default_rng(seed)
    th = (rng.standard_normal(S.param_count(cfg)) * spread).astype(dtype)
    for name, off, r, c in S.param_layout(cfg):
        if name.endswith(".g"):
            th[off:off + r * c] += 1.0
    return th


def _batch(seed, src_lens=(5, 8, 3), tgt_lens=(6, 4, 8), Ls=8, Lt=8, vocab=31):
    return synth.make_pair_batch(np.random.default_rng(seed), src_lens, tgt_lens, Ls, Lt, vocab, "uniform")


def _loss(cfg, th, mb, eps=0.1):
    y, cache = S.forward(cfg, th, mb["src"], mb["src_lens"], mb["tgt_in"], mb["tgt_lens"], mb.get("drop"))
    g = np.zeros_like(th)
    return S.loss_forward_backward(cfg, th, y, mb["tgt_out"], mb["tgt_lens"], eps, g)[0]


@pytest.mark.parametrize("dropout", [0.0, 0.25])
def test_gradient_matches_central_differences_for_every_tensor(dropout):
    mb = _batch(1)
    if dropout:
        mb["drop"] = dict(p=dropout, seed=11, stream=3)
    th = _theta(CFG, 2)
    loss, nll, grad, n_seq, n_tok = S.micro_batch_grad(CFG, th, mb, 0.1)
    assert n_seq == 3 and n_tok == 18
    rng = np.random.default_rng(3)
    h = 1e-5
    for name, off, r, c in S.param_layout(CFG):
        for k in rng.choice(r * c, size=min(4, r * c), replace=False):
            tp, tm = th.copy(), th.copy()
            tp[off + k] += h
            tm[off + k] -= h
            fd = (_loss(CFG, tp, mb) - _loss(CFG, tm, mb)) / (2 * h)
            assert abs(fd - grad[off + k]) <= 1e-6 * max(1.0, abs(fd)), (name, k, fd, grad[off + k])


def test_attention_equals_a_python_loop_over_allowed_pairs():
    rng = np.random.default_rng(4)
    B, Lq, Lk, A, d = 2, 5, 7, 2, 3
    q, k, v = (rng.standard_normal((B, L, A * d)) for L in (Lq, Lk, Lk))
    for causal, klens in ((False, [7, 4]), (True, [5, 3])):
        Lk_ = Lk if not causal else Lq
        kk, vv = k[:, :Lk_], v[:, :Lk_]
        ok = S.allowed_pairs(Lq, klens, Lk_, causal)
        ctx, _ = S.attention_forward(q, kk, vv, ok, A)
        for b in range(B):
            for h in range(A):
                for i in range(Lq):
                    js = [j for j in range(Lk_) if j < klens[b] and (not causal or j <= i)]
                    sc = [sum(q[b, i, h * d + c] * kk[b, j, h * d + c] for c in range(d)) / math.sqrt(d) for j in js]
                    m = max(sc)
                    w = [math.exp(s - m) for s in sc]
                    for c in range(d):
                        want = sum(wj * vv[b, j, h * d + c] for wj, j in zip(w, js)) / sum(w)
                        assert abs(ctx[b, i, h * d + c] - want) < 1e-12


def test_decoder_is_causal_and_ignores_padding():
    th = _theta(CFG, 5)
    mb = _batch(6)
    y, _ = S.forward(CFG, th, mb["src"], mb["src_lens"], mb["tgt_in"], mb["tgt_lens"])
    # a later target token changes no earlier output position
    t2 = mb["tgt_in"].copy()
    t2[:, 4] = (t2[:, 4] + 7) % 26 + 5
    y2, _ = S.forward(CFG, th, mb["src"], mb["src_lens"], t2, mb["tgt_lens"])
    assert np.array_equal(y[:, :4], y2[:, :4]) and not np.allclose(y[:, 4:], y2[:, 4:])
    # tokens in the padding of either side change nothing that counts
    s3, t3 = mb["src"].copy(), mb["tgt_in"].copy()
    for b in range(3):
        s3[b, mb["src_lens"][b]:] = 9
        t3[b, mb["tgt_lens"][b]:] = 9
    a = S.micro_batch_grad(CFG, th, mb)
    b_ = S.micro_batch_grad(CFG, th, dict(mb, src=s3, tgt_in=t3))
    assert abs(a[0] - b_[0]) < 1e-12 and np.allclose(a[2], b_[2], rtol=0, atol=1e-12)


def test_padding_to_longer_buffers_changes_neither_loss_nor_gradient():
    th = _theta(CFG, 7)
    mb = _batch(8)
    wide = dict(mb)
    for k, pad in (("src", 4), ("tgt_in", 8), ("tgt_out", 8)):
        wide[k] = np.pad(mb[k], ((0, 0), (0, pad)))
    a, b = S.micro_batch_grad(CFG, th, mb), S.micro_batch_grad(CFG, th, wide)
    assert abs(a[0] - b[0]) < 1e-11 and a[4] == b[4]
    assert np.allclose(a[2], b[2], rtol=0, atol=1e-11)
    # and a batch is the sum of its sentences run alone (no interaction across sequences)
    tot = np.zeros_like(th)
    ls = 0.0
    for i in range(3):
        one = {k: (v[i:i + 1] if isinstance(v, np.ndarray) else v) for k, v in mb.items()}
        r = S.micro_batch_grad(CFG, th, one)
        tot += r[2]
        ls += r[0]
    assert abs(ls - a[0]) < 1e-11 and np.allclose(tot, a[2], rtol=0, atol=1e-11)


def test_label_smoothing_is_cross_entropy_to_the_mixed_target():
    rng = np.random.default_rng(9)
    T, V, eps = 6, 11, 0.1
    z = rng.standard_normal((T, V)) * 2
    lab = np.array([3, -1, 0, 10, 5, -1])
    loss, nll, d = S.smoothed_ce(z, lab, eps)
    logp = z - logsumexp(z, axis=1, keepdims=True)
    want = want_nll = 0.0
    for t in range(T):
        if lab[t] < 0:
            assert not d[t].any()
            continue
        qd = np.full(V, eps / V)
        qd[lab[t]] += 1 - eps
        want += -(qd * logp[t]).sum()
        want_nll += -logp[t, lab[t]]
        assert np.allclose(d[t], np.exp(logp[t]) - qd, atol=1e-14)       # gradient of CE(q, softmax z) is p - q
    assert abs(loss - want) < 1e-12 and abs(nll - want_nll) < 1e-12
    # eps = 0 is the plain negative log-likelihood; uniform logits give ln V whatever eps is
    assert abs(S.smoothed_ce(z, lab, 0.0)[0] - want_nll) < 1e-12
    assert abs(S.smoothed_ce(np.zeros((2, V)), [1, 2], 0.3)[0] - 2 * math.log(V)) < 1e-12


def test_positional_table_closed_forms():
    pe = S.positional_table(50, 8)
    assert np.array_equal(pe[0], [0, 1, 0, 1, 0, 1, 0, 1])
    assert np.allclose(pe[:, 0], np.sin(np.arange(50))) and np.allclose(pe[:, 1], np.cos(np.arange(50)))
    # pair i has wavelength 2 pi 10000^(2i/H): the last pair of H = 8 turns once in 2 pi 10000^(6/8) positions
    assert np.allclose(pe[:, 6], np.sin(np.arange(50) / 10000 ** 0.75))
    assert np.allclose(pe[:, 0::2] ** 2 + pe[:, 1::2] ** 2, 1.0)


def test_attention_over_one_key_returns_its_value():
    rng = np.random.default_rng(10)
    q, k, v = rng.standard_normal((2, 4, 6)), rng.standard_normal((2, 1, 6)), rng.standard_normal((2, 1, 6))
    ctx, cache = S.attention_forward(q, k, v, S.allowed_pairs(4, [1, 1], 1, False), 2)
    assert np.allclose(ctx, np.broadcast_to(v, ctx.shape))
    dq, dk, dv = S.attention_backward(np.ones_like(ctx), cache, 2)
    assert np.allclose(dq, 0) and np.allclose(dk, 0) and np.allclose(dv, 4.0)


def test_base_model_has_about_65_million_parameters():
    n = S.param_count(S.S2SCfg(**synth.S2S_MODELS["transformer_base"]))
    assert n == 37000 * 512 + 6 * (4 * 512 * 512 + 2 * 512 * 2048 + 9 * 512 + 2048) + 6 * (8 * 512 * 512 + 2 * 512 * 2048 + 15 * 512 + 2048)
    assert 60e6 < n < 66e6     # section "Transformer Translation Model": about 65 million


def test_first_loss_is_near_ln_v_at_small_initial_weights():
    cfg = S.S2SCfg(**synth.S2S_MODELS["s2s_tiny"])
    th = synth.init_params(S.param_layout(cfg), 1).astype(np.float64)
    mb = synth.make_pair_batch(synth.rng_for(2), [9, 16], [12, 7], 16, 16, cfg.vocab, "uniform")
    loss, nll, g, n_seq, n_tok = S.micro_batch_grad(cfg, th, mb)
    assert abs(nll / n_tok - math.log(cfg.vocab)) < 0.5
