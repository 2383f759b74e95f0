"""Pins of the CPU oracle to things other than itself (CPU only).

Each test fixes the oracle against a closed form, an invariant, a library routine, brute
force, or a value the paper prints (tests/golden/*.txt).
"""
import math
import os

import numpy as np
import pytest
from scipy.special import logsumexp

from oracle import hetseq_oracle as O
from paper_2009_14783_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, *v = line.split()
            out[k] = v
    return out


MICRO = O.ModelCfg(n_layers=2, hidden=16, n_heads=2, ffn=32, vocab=29, max_pos=8, ln_eps=1e-12)


def micro_theta(cfg, seed, std=0.3, dtype=np.float64):
    rng = np.random.default_rng(seed)
    th = rng.standard_normal(O.param_count(cfg)) * std
    for name, off, r, c in O.param_layout(cfg):
        if name.endswith(".g"):
            th[off:off + r * c] += 1.0
    return th.astype(dtype)


def micro_batch(cfg, lens, L, seed):
    return synth.make_micro_batch(synth.rng_for(seed), lens, L, cfg.vocab, "uniform")


def loss_of(cfg, theta, mb):
    hidden, _ = O.encoder_forward(cfg, theta, mb["ids"], mb["lens"])
    loss, _ = O.mlm_loss_forward(cfg, theta, hidden, mb["mlm_pos"], mb["mlm_label"])
    return float(loss)


# ---------------------------------------------------------------- layout
def test_param_counts_match_published_model_sizes():
    tiny = O.ModelCfg(**synth.MODELS["tiny"])
    base = O.ModelCfg(**synth.MODELS["bert_base"])
    large = O.ModelCfg(**synth.MODELS["bert_large"])
    assert O.param_count(tiny) == 352_488
    # BERT-base without token-type embeddings / pooler: 109.5 M
    assert O.param_count(base) == 109_512_762
    assert O.param_count(large) == 335_172_410
    lay = O.param_layout(base)
    offs = [o for _, o, _, _ in lay]
    assert offs == sorted(offs) and offs[0] == 0
    for (_, o, r, c), (_, o2, _, _) in zip(lay[:-1], lay[1:]):
        assert o + r * c == o2


# ---------------------------------------------------------------- elementary pieces
def test_gelu_closed_values():
    # GELU(x) = x * Phi(x); Phi(1) = 0.841344746068543, Phi(-2) = 0.022750131948179
    x = np.array([0.0, 1.0, -2.0, 6.0, -9.0])
    want = np.array([0.0, 0.841344746068543, -2.0 * 0.022750131948179, 6.0 * (1 - 9.8658764503769e-10), 0.0])
    np.testing.assert_allclose(O.gelu(x), want, rtol=1e-12, atol=1e-15)
    h = 1e-6
    xs = np.linspace(-4, 4, 41)
    fd = (O.gelu(xs + h) - O.gelu(xs - h)) / (2 * h)
    np.testing.assert_allclose(O.gelu_grad(xs), fd, rtol=1e-8, atol=1e-9)


def test_layer_norm_statistics_and_affine():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 7, 16)) * 3 + 2
    y, _ = O.layer_norm_fwd(x, np.ones(16), np.zeros(16), 0.0)
    np.testing.assert_allclose(y.mean(-1), 0, atol=1e-13)
    np.testing.assert_allclose((y * y).mean(-1), 1, rtol=1e-12)       # biased variance
    g, b = rng.standard_normal(16), rng.standard_normal(16)
    y2, _ = O.layer_norm_fwd(x, g, b, 0.0)
    np.testing.assert_allclose(y2, y * g + b, rtol=1e-12, atol=1e-12)
    # invariance to shift and positive scale of the input
    y3, _ = O.layer_norm_fwd(4.0 * x + 11.0, np.ones(16), np.zeros(16), 0.0)
    np.testing.assert_allclose(y3, y, rtol=1e-10, atol=1e-10)


def test_loss_is_logsumexp_minus_target_logit():
    cfg = MICRO
    th = micro_theta(cfg, 3)
    mb = micro_batch(cfg, [8, 3, 5], 8, 7)
    hidden, _ = O.encoder_forward(cfg, th, mb["ids"], mb["lens"])
    loss, c = O.mlm_loss_forward(cfg, th, hidden, mb["mlm_pos"], mb["mlm_label"])
    want = (logsumexp(c["logits"], axis=1) - c["logits"][np.arange(c["M"]), mb["mlm_label"]]).sum()
    assert abs(loss - want) <= 1e-12 * abs(want)
    # cross-entropy of a uniform distribution over V classes is ln V per target
    th0 = np.zeros_like(th)
    for name, off, r, cc in O.param_layout(cfg):
        if name.endswith(".g"):
            th0[off:off + r * cc] = 1.0
    assert abs(loss_of(cfg, th0, mb) - c["M"] * math.log(cfg.vocab)) < 1e-10


def test_loss_near_ln_vocab_at_small_init():
    cfg = O.ModelCfg(**synth.MODELS["tiny"])
    th = synth.init_params(O.param_layout(cfg), 1234)
    mb = synth.workload_micro_batches(0)[0]
    assert mb["mlm_pos"].size == 24 and mb["n_real_tokens"] == 160     # lens 16/32/48/64 -> 2+5+7+10
    per_tok = loss_of(cfg, th, mb) / mb["mlm_pos"].size
    assert abs(per_tok - math.log(1000)) < 0.05


# ---------------------------------------------------------------- brute force forward
def naive_forward_loss(cfg, theta, ids, lens, mlm_pos, mlm_label):
    """Pure-Python loops, no NumPy linear algebra: index-by-index statement of the model."""
    P = {k: v.tolist() for k, v in O.param_views(cfg, theta).items()}
    B, L = ids.shape
    H, A, d, F, V = cfg.hidden, cfg.n_heads, cfg.head_dim, cfg.ffn, cfg.vocab

    def ln(vec, g, b):
        mu = sum(vec) / len(vec)
        var = sum((t - mu) ** 2 for t in vec) / len(vec)
        return [(t - mu) / math.sqrt(var + cfg.ln_eps) * g[j] + b[j] for j, t in enumerate(vec)]

    def lin(vec, W, b):                       # W[out][in]
        return [sum(W[o][i] * vec[i] for i in range(len(vec))) + b[o] for o in range(len(W))]

    def gelu(t):
        return 0.5 * t * (1.0 + math.erf(t / math.sqrt(2.0)))

    hidden = []
    for bi in range(B):
        x = [ln([P["emb.word"][ids[bi, l]][j] + P["emb.pos"][l][j] for j in range(H)],
                P["emb.ln.g"], P["emb.ln.b"]) for l in range(L)]
        for i in range(cfg.n_layers):
            p = f"l{i}."
            qkv = [lin(x[l], P[p + "qkv.w"], P[p + "qkv.b"]) for l in range(L)]
            ctx = [[0.0] * H for _ in range(L)]
            for a in range(A):
                for l in range(L):
                    sc = []
                    for l2 in range(int(lens[bi])):               # only real keys
                        sc.append(sum(qkv[l][a * d + c] * qkv[l2][H + a * d + c] for c in range(d)) / math.sqrt(d))
                    mx = max(sc)
                    ex = [math.exp(t - mx) for t in sc]
                    z = sum(ex)
                    for c in range(d):
                        ctx[l][a * d + c] = sum(ex[l2] / z * qkv[l2][2 * H + a * d + c] for l2 in range(len(sc)))
            x1 = []
            for l in range(L):
                o = lin(ctx[l], P[p + "o.w"], P[p + "o.b"])
                x1.append(ln([x[l][j] + o[j] for j in range(H)], P[p + "ln1.g"], P[p + "ln1.b"]))
            x2 = []
            for l in range(L):
                hh = [gelu(t) for t in lin(x1[l], P[p + "ffn1.w"], P[p + "ffn1.b"])]
                o = lin(hh, P[p + "ffn2.w"], P[p + "ffn2.b"])
                x2.append(ln([x1[l][j] + o[j] for j in range(H)], P[p + "ln2.g"], P[p + "ln2.b"]))
            x = x2
        hidden.append(x)
    loss = 0.0
    for pos, lab in zip(mlm_pos.tolist(), mlm_label.tolist()):
        row = hidden[pos // L][pos % L]
        t = ln([gelu(u) for u in lin(row, P["head.t.w"], P["head.t.b"])], P["head.ln.g"], P["head.ln.b"])
        logits = [sum(P["emb.word"][v][j] * t[j] for j in range(H)) + P["head.dec.b"][v] for v in range(V)]
        mx = max(logits)
        loss += mx + math.log(sum(math.exp(u - mx) for u in logits)) - logits[lab]
    return loss, hidden


def test_forward_matches_pure_python_loops():
    cfg = MICRO
    th = micro_theta(cfg, 11)
    mb = micro_batch(cfg, [8, 3, 5], 8, 5)
    want, hid = naive_forward_loss(cfg, th, mb["ids"], mb["lens"], mb["mlm_pos"], mb["mlm_label"])
    got = loss_of(cfg, th, mb)
    assert abs(got - want) <= 1e-11 * abs(want)
    hidden, _ = O.encoder_forward(cfg, th, mb["ids"], mb["lens"])
    valid = O.key_mask(mb["lens"], 8).astype(bool)
    np.testing.assert_allclose(hidden[valid], np.array(hid)[valid], rtol=1e-10, atol=1e-12)


def test_attention_special_cases():
    # one real key: every head's context is that key's value vector, whatever the scores
    cfg = O.ModelCfg(n_layers=1, hidden=16, n_heads=2, ffn=32, vocab=29, max_pos=8)
    th = micro_theta(cfg, 2)
    ids = np.array([[7, 0, 0, 0]], dtype=np.int32)
    _, cache = O.encoder_forward(cfg, th, ids, np.array([1]))
    c = cache["layers"][0]
    v0 = c["v"][0, :, 0, :].reshape(-1)
    np.testing.assert_allclose(c["ctx"][0, 0], v0, rtol=1e-12)
    assert np.all(c["prob"][0, :, :, 1:] == 0.0)
    np.testing.assert_allclose(c["prob"].sum(-1), 1.0, rtol=1e-12)


def test_key_mask_definition():
    m = O.key_mask(np.array([1, 3, 4]), 4)
    assert m.dtype == np.uint8
    assert m.tolist() == [[1, 0, 0, 0], [1, 1, 1, 0], [1, 1, 1, 1]]


# ---------------------------------------------------------------- backward: finite differences
def test_gradients_match_central_finite_differences_fp64():
    cfg = MICRO
    th = micro_theta(cfg, 21)
    mb = micro_batch(cfg, [8, 3, 5], 8, 9)
    # make sure at least one token id repeats (embedding scatter must sum duplicates)
    assert len(set(mb["ids"].reshape(-1).tolist())) < mb["ids"].size
    loss, grad, n_seq, n_tok = O.micro_batch_grad(cfg, th, mb["ids"], mb["lens"], mb["mlm_pos"], mb["mlm_label"])
    assert n_seq == 3 and n_tok == mb["mlm_pos"].size
    rng = np.random.default_rng(4)
    eps = 1e-5
    for name, off, r, c in O.param_layout(cfg):
        n = r * c
        # random direction confined to this tensor
        u = np.zeros_like(th)
        u[off:off + n] = rng.standard_normal(n)
        fd = (loss_of(cfg, th + eps * u, mb) - loss_of(cfg, th - eps * u, mb)) / (2 * eps)
        an = float(grad @ u)
        assert abs(fd - an) <= 1e-6 * max(abs(fd), abs(an)) + 1e-9, (name, fd, an)
        # and three single entries
        for j in rng.choice(n, size=min(3, n), replace=False):
            e = np.zeros_like(th)
            e[off + j] = 1.0
            fd1 = (loss_of(cfg, th + eps * e, mb) - loss_of(cfg, th - eps * e, mb)) / (2 * eps)
            assert abs(fd1 - grad[off + j]) <= 1e-6 * max(abs(fd1), abs(grad[off + j])) + 1e-8, (name, j)


def test_fp32_oracle_agrees_with_fp64_oracle():
    cfg = O.ModelCfg(**synth.MODELS["tiny"])
    th = synth.init_params(O.param_layout(cfg), 1234)
    mb = synth.workload_micro_batches(0)[0]
    l32, g32, _, _ = O.micro_batch_grad(cfg, th, mb["ids"], mb["lens"], mb["mlm_pos"], mb["mlm_label"])
    l64, g64, _, _ = O.micro_batch_grad(cfg, th.astype(np.float64), mb["ids"], mb["lens"], mb["mlm_pos"], mb["mlm_label"])
    assert g32.dtype == np.float32
    assert abs(l32 - l64) <= 2e-6 * abs(l64)
    for name, off, r, c in O.param_layout(cfg):
        a, b = g32[off:off + r * c].astype(np.float64), g64[off:off + r * c]
        assert np.linalg.norm(a - b) <= 2e-5 * np.linalg.norm(b) + 1e-12, name


# ---------------------------------------------------------------- invariants
def test_padding_invariance():
    """Parameter gradients do not depend on padding: a padded batch equals the sum of its
    sequences run alone without padding, and the same batch padded further."""
    cfg = MICRO
    th = micro_theta(cfg, 31)
    mb = micro_batch(cfg, [2, 7, 4], 8, 13)
    loss, grad, _, _ = O.micro_batch_grad(cfg, th, mb["ids"], mb["lens"], mb["mlm_pos"], mb["mlm_label"])
    tot_l, tot_g = 0.0, np.zeros_like(th)
    for b, n in enumerate(mb["lens"]):
        sel = (mb["mlm_pos"] // 8) == b
        l1, g1, _, _ = O.micro_batch_grad(cfg, th, mb["ids"][b:b + 1, :n], [n],
                                          mb["mlm_pos"][sel] - b * 8, mb["mlm_label"][sel])
        tot_l += l1
        tot_g += g1
    assert abs(tot_l - loss) <= 1e-12 * abs(loss)
    np.testing.assert_allclose(tot_g, grad, rtol=1e-9, atol=1e-12)
    # narrower padding (7 instead of 8)
    ids7 = mb["ids"][:, :7]
    pos7 = (mb["mlm_pos"] // 8) * 7 + mb["mlm_pos"] % 8
    l7, g7, _, _ = O.micro_batch_grad(cfg, th, ids7, mb["lens"], pos7, mb["mlm_label"])
    assert abs(l7 - loss) <= 1e-12 * abs(loss)
    np.testing.assert_allclose(g7, grad, rtol=1e-9, atol=1e-12)


def test_padded_positions_receive_no_gradient():
    cfg = MICRO
    th = micro_theta(cfg, 33)
    mb = micro_batch(cfg, [2, 7, 4], 8, 15)
    hidden, cache = O.encoder_forward(cfg, th, mb["ids"], mb["lens"])
    _, hc = O.mlm_loss_forward(cfg, th, hidden, mb["mlm_pos"], mb["mlm_label"])
    grad = np.zeros_like(th)
    dh = O.mlm_loss_backward(cfg, th, hidden.shape, hc, grad)
    on = np.zeros(hidden.shape[:2], dtype=bool).reshape(-1)
    on[mb["mlm_pos"]] = True
    assert np.all(dh.reshape(-1, cfg.hidden)[~on] == 0.0)
    enc_only = np.zeros_like(th)
    O.encoder_backward(cfg, th, cache, dh, enc_only)
    # through the encoder, the PAD row of the word embedding sees only padded positions -> exactly
    # zero (the tied decoder's contribution to that row lives in `grad`, not here)
    assert np.all(O.param_views(cfg, enc_only)["emb.word"][synth.PAD_ID] == 0.0)
    assert np.any(O.param_views(cfg, enc_only)["emb.word"][synth.MASK_ID] != 0.0)


def test_concatenation_invariant_unequal_micro_batches():
    """Summing the gradients of unequal micro-batches and dividing by the global sample
    count equals the gradient of the one concatenated batch divided by the same count."""
    cfg = MICRO
    th = micro_theta(cfg, 41)
    rng = synth.rng_for(77)
    mbs = [synth.make_micro_batch(rng, lens, 8, cfg.vocab, "uniform")
           for lens in ([8, 5], [3, 8, 8, 6, 2, 7], [4] * 14)]             # shares 2 : 6 : 14
    G, n = np.zeros_like(th), 0
    loss_total = 0.0
    for mb in mbs:
        l, g, ns, _ = O.micro_batch_grad(cfg, th, mb["ids"], mb["lens"], mb["mlm_pos"], mb["mlm_label"])
        G, n = O.accumulate(G, n, g, ns)
        loss_total += l
    assert n == 22
    O.normalize(G, n)
    big = synth.concat_micro_batches(mbs)
    lb, gb, nb, _ = O.micro_batch_grad(cfg, th, big["ids"], big["lens"], big["mlm_pos"], big["mlm_label"])
    assert nb == 22
    np.testing.assert_allclose(G, gb / 22, rtol=1e-9, atol=1e-13)
    assert abs(loss_total - lb) <= 1e-12 * abs(lb)


def test_paper_worked_example_weights_2_2_1_0():
    """Five instances over four workers with local batches 2, 2, 1, 0: the weighted
    aggregation equals the single five-instance average, a plain mean of the per-worker
    mean losses does not, and the empty worker contributes nothing."""
    gold = read_golden("paper_worked_example.txt")
    local = [int(t) for t in gold["local_batches"]]
    assert local == [2, 2, 1, 0] and sum(local) == int(gold["instances"][0])
    assert len(local) == int(gold["workers"][0]) and max(local) == int(gold["global_batch"][0])
    cfg = MICRO
    th = micro_theta(cfg, 51)
    rng = synth.rng_for(5)
    seqs = [synth.make_micro_batch(rng, [n], 8, cfg.vocab, "uniform") for n in (8, 6, 7, 3, 5)]
    shares, k = [], 0
    for nloc in local:
        shares.append(synth.concat_micro_batches(seqs[k:k + nloc]) if nloc else None)
        k += nloc
    G, n, loss_sum, mean_of_means = np.zeros_like(th), 0, 0.0, []
    grads_mean = np.zeros_like(th)
    for sh in shares:
        if sh is None:                                 # worker D: dummy batch, zero gradient
            G, n = O.accumulate(G, n, None, 0, ignore=True)
            continue
        l, g, ns, _ = O.micro_batch_grad(cfg, th, sh["ids"], sh["lens"], sh["mlm_pos"], sh["mlm_label"])
        G, n = O.accumulate(G, n, g, ns)
        loss_sum += l
        mean_of_means.append(l / ns)
        grads_mean += g / ns
    assert n == 5
    O.normalize(G, n)
    allfive = synth.concat_micro_batches(seqs)
    l5, g5, _, _ = O.micro_batch_grad(cfg, th, allfive["ids"], allfive["lens"], allfive["mlm_pos"], allfive["mlm_label"])
    np.testing.assert_allclose(G, g5 / 5, rtol=1e-9, atol=1e-13)
    assert abs(loss_sum / 5 - l5 / 5) < 1e-12 * abs(l5)
    # the unweighted alternatives are NOT equivalent
    assert abs(np.mean(mean_of_means) - l5 / 5) > 1e-3 * abs(l5 / 5)
    assert np.linalg.norm(grads_mean / 4 - g5 / 5) > 1e-3 * np.linalg.norm(g5 / 5)


def test_delayed_update_equals_workers():
    """k accumulation passes on one worker equal k workers with one pass each: the
    accumulate/normalise result does not depend on how the micro-batches are grouped."""
    gold = read_golden("paper_delayed_update.txt")
    k = int(gold["steps_on_one_gpu"][0])
    assert k == int(gold["gpus"][0]) == 16
    rng = np.random.default_rng(0)
    gs = [rng.standard_normal(50) for _ in range(k)]
    ns = [int(t) for t in rng.integers(1, 9, size=k)]
    G1, n1 = np.zeros(50), 0
    for g, n in zip(gs, ns):                           # one worker, 16 passes
        G1, n1 = O.accumulate(G1, n1, g, n)
    O.normalize(G1, n1)
    Gk = np.sum(gs, axis=0) / sum(ns)                  # 16 workers, one exchange
    np.testing.assert_allclose(G1, Gk, rtol=1e-12)


def test_dummy_batch_leaves_buffer_and_count_bit_identical():
    rng = np.random.default_rng(1)
    G = rng.standard_normal(100).astype(np.float32)
    before = G.copy()
    poison = np.full(100, np.nan, dtype=np.float32)
    G2, n2 = O.accumulate(G, 7, poison, 3, ignore=True)
    assert n2 == 7 and G2.tobytes() == before.tobytes()


# ---------------------------------------------------------------- Adam
def test_adam_closed_forms_and_paper_hyperparameters():
    gold = read_golden("paper_adam_bert.txt")
    b1, b2 = float(gold["beta1"][0]), float(gold["beta2"][0])
    eps, lr = float(gold["eps"][0]), float(gold["max_lr"][0])
    assert (b1, b2, eps, lr) == (0.9, 0.999, 1e-8, 1e-4)
    rng = np.random.default_rng(2)
    g = rng.standard_normal(64)
    g[:4] = [0.0, 1e-3, -2.5, 7.0]
    # first step from zero state: delta = -lr * g / (|g| + eps)
    w0 = rng.standard_normal(64)
    w, m, v = w0.copy(), np.zeros(64), np.zeros(64)
    O.adam_step(w, m, v, g, 1, lr, b1, b2, eps)
    np.testing.assert_allclose(w - w0, -lr * g / (np.abs(g) + eps), rtol=1e-9, atol=1e-18)
    np.testing.assert_allclose(m, (1 - b1) * g, rtol=1e-12)
    np.testing.assert_allclose(v, (1 - b2) * g * g, rtol=1e-12)
    # a constant gradient gives the same delta at every step
    prev = w.copy()
    for t in range(2, 6):
        O.adam_step(w, m, v, g, t, lr, b1, b2, eps)
        np.testing.assert_allclose(w - prev, -lr * g / (np.abs(g) + eps), rtol=1e-7, atol=1e-18)
        prev = w.copy()
    # textbook recurrence written with scalars, two different gradients
    ww, mm, vv = 0.3, 0.0, 0.0
    w1, m1, v1 = np.array([0.3]), np.zeros(1), np.zeros(1)
    for t, gg in enumerate([0.5, -0.2, 0.9], start=1):
        mm = b1 * mm + (1 - b1) * gg
        vv = b2 * vv + (1 - b2) * gg * gg
        ww -= lr * (mm / (1 - b1 ** t)) / (math.sqrt(vv / (1 - b2 ** t)) + eps)
        O.adam_step(w1, m1, v1, np.array([gg]), t, lr, b1, b2, eps)
        assert abs(w1[0] - ww) < 1e-15
    # decoupled weight decay
    w2, m2, v2 = np.array([2.0]), np.zeros(1), np.zeros(1)
    O.adam_step(w2, m2, v2, np.array([0.0]), 1, 0.1, b1, b2, eps, weight_decay=0.5)
    assert abs(w2[0] - (2.0 - 0.1 * 0.5 * 2.0)) < 1e-15


def test_train_step_reports_weighted_loss_and_updates_once():
    cfg = MICRO
    th = micro_theta(cfg, 61)
    rng = synth.rng_for(9)
    mbs = [synth.make_micro_batch(rng, lens, 8, cfg.vocab, "uniform") for lens in ([8, 5], [3, 8, 6])]
    mbs.insert(1, dict(dummy=True))
    th1, m, v = th.copy(), np.zeros_like(th), np.zeros_like(th)
    loss, G, D = O.train_step(cfg, th1, m, v, 1, mbs, lr=1e-3, eps=1e-8)
    assert D == 5
    big = synth.concat_micro_batches([mbs[0], mbs[2]])
    lb, gb, _, _ = O.micro_batch_grad(cfg, th, big["ids"], big["lens"], big["mlm_pos"], big["mlm_label"])
    assert abs(loss - lb / 5) < 1e-12 * abs(lb)
    np.testing.assert_allclose(G, gb / 5, rtol=1e-9, atol=1e-13)
    np.testing.assert_allclose(th1 - th, -1e-3 * G / (np.abs(G) + 1e-8), rtol=1e-7, atol=1e-16)


# ---------------------------------------------------------------- schedule and loop
def test_lr_schedule_paper_settings_and_linearity():
    rows = []
    par = {}
    with open(os.path.join(GOLDEN, "paper_lr_schedule.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = line.split()
            if k in ("max_lr", "warmup", "total"):
                par[k] = float(v) if k == "max_lr" else int(v)
            else:
                rows.append((int(k), float(v)))
    assert par == dict(max_lr=1e-4, warmup=10000, total=1000000)
    for t, want in rows:
        got = O.lr_linear(t, **par)
        assert got == pytest.approx(want, rel=1e-12, abs=1e-20), (t, got, want)
    # straight lines: constant first differences inside each segment, continuous at the junction,
    # never above the maximum, zero at and beyond the end
    lr = np.array([O.lr_linear(t, 3e-4, 7, 40) for t in range(1, 46)])
    up, down = np.diff(lr[:7]), np.diff(lr[6:40])
    assert np.allclose(up, 3e-4 / 7, rtol=1e-12) and np.allclose(down, -3e-4 / 33, rtol=1e-12)
    assert lr[6] == 3e-4 and lr.max() == 3e-4 and np.all(lr[39:] == 0.0)
    # no warm-up: the first update already decays from the maximum
    assert O.lr_linear(1, 1.0, 0, 10) == pytest.approx(0.9)
    with pytest.raises(ValueError):
        O.lr_linear(0, 1.0, 2, 10)


def test_train_loop_wires_schedule_and_update_number():
    cfg = MICRO
    adam = dict(beta1=0.9, beta2=0.999, eps=1e-12)
    sched = dict(max_lr=1e-3, warmup=4, total=12)
    batches = lambda t: [micro_batch(cfg, [8, 5, 3], 8, 1000 + t)]
    th0 = micro_theta(cfg, 3)
    st = dict(theta=th0.copy(), m=np.zeros_like(th0), v=np.zeros_like(th0), step=0)
    O.train_loop(cfg, st, 1, batches, adam, sched)
    # First Adam update with bias correction moves every parameter with a non-zero gradient by
    # exactly the learning rate (m_hat / sqrt(v_hat) = +-1): here lr(1) = max_lr / warmup.
    step = np.abs(st["theta"] - th0)
    moved = step > 0
    assert moved.sum() > 0.9 * th0.size
    lr1 = 1e-3 / 4
    assert np.all(step <= lr1 * (1 + 1e-9))                      # (entries with |g| near eps move a little less)
    assert np.mean(np.abs(step[moved] - lr1) <= 1e-6 * lr1) > 0.99
    assert st["step"] == 1
    # a zero maximum rate changes nothing but still counts updates
    st2 = dict(theta=th0.copy(), m=np.zeros_like(th0), v=np.zeros_like(th0), step=0)
    O.train_loop(cfg, st2, 3, batches, adam, dict(max_lr=0.0, warmup=4, total=12))
    assert np.array_equal(st2["theta"], th0) and st2["step"] == 3
    # the loss on a repeated batch goes down over a few updates
    st3 = dict(theta=th0.copy(), m=np.zeros_like(th0), v=np.zeros_like(th0), step=0)
    same = lambda t: [micro_batch(cfg, [8, 5, 3], 8, 77)]
    losses = O.train_loop(cfg, st3, 8, same, adam, dict(max_lr=3e-2, warmup=2, total=40))
    assert losses[-1] < losses[0] - 0.1


def test_train_loop_resumed_equals_uninterrupted():
    cfg = MICRO
    adam = dict(beta1=0.9, beta2=0.999, eps=1e-8)
    sched = dict(max_lr=2e-3, warmup=3, total=10)
    batches = lambda t: synth.step_micro_batches(42, t, [8, 6, 2], 8, cfg.vocab, "uniform", n_micro=2)
    th0 = micro_theta(cfg, 9, dtype=np.float32)
    full = dict(theta=th0.copy(), m=np.zeros_like(th0), v=np.zeros_like(th0), step=0)
    l_full = O.train_loop(cfg, full, 7, batches, adam, sched)
    part = dict(theta=th0.copy(), m=np.zeros_like(th0), v=np.zeros_like(th0), step=0)
    l_a = O.train_loop(cfg, part, 3, batches, adam, sched)
    snap = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in part.items()}   # the checkpoint
    l_b = O.train_loop(cfg, snap, 4, batches, adam, sched)
    assert l_a + l_b == l_full
    for k in ("theta", "m", "v"):
        assert np.array_equal(snap[k], full[k])
    assert snap["step"] == full["step"] == 7


# ---------------------------------------------------------------- dropout
def test_philox_known_answers():
    with open(os.path.join(GOLDEN, "philox4x32_10_known_answers.txt")) as f:
        rows = [line.split() for line in f if line.strip() and not line.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        w = [int(x, 16) for x in r]
        out = O.philox4x32_10(np.array([w[:4]], dtype=np.uint32), (w[4], w[5]))[0]
        assert [int(x) for x in out] == w[6:], r
    # vectorised calls give what single calls give
    ctr = np.arange(40, dtype=np.uint32).reshape(10, 4)
    many = O.philox4x32_10(ctr, (7, 9))
    for i in range(10):
        assert np.array_equal(many[i], O.philox4x32_10(ctr[i:i + 1], (7, 9))[0])


def test_dropout_mask_properties():
    drop = dict(p=0.1, seed=0x1234567890ABCDEF, stream=3)
    n = 400_003                                             # not a multiple of 4
    keep = O.dropout_keep(drop, 5, n)
    assert keep.shape == (n,)
    # drop frequency within 5 standard deviations of p
    assert abs((~keep).mean() - 0.1) < 5 * math.sqrt(0.1 * 0.9 / n)
    # a prefix of a longer site is the same mask (element e depends on e, site, stream, seed only)
    assert np.array_equal(O.dropout_keep(drop, 5, 1001), keep[:1001])
    # other site, stream or seed: another mask, and (nearly) independent of this one
    for other in (O.dropout_keep(drop, 6, n), O.dropout_keep(dict(drop, stream=4), 5, n), O.dropout_keep(dict(drop, seed=1), 5, n)):
        both = (~keep & ~other).mean()
        assert abs(both - 0.01) < 5 * math.sqrt(0.01 * 0.99 / n)
    # thresholds at the ends
    assert O.dropout_keep(dict(drop, p=0.0), 0, 1000).all()
    assert (~O.dropout_keep(dict(drop, p=1.0 - 2.0 ** -33), 0, 100000)).mean() > 0.9999
    # exactly the definition for one element: word e % 4 of block e // 4
    e = 123457
    blk = O.philox4x32_10(np.array([[e // 4, 0, 5, 3]], dtype=np.uint32), (0x90ABCDEF, 0x12345678))[0]
    assert keep[e] == (int(blk[e % 4]) >= int(math.floor(0.1 * 2 ** 32)))


def test_dropout_is_unbiased_and_identity_at_zero():
    x = np.linspace(-2.0, 3.0, 64).reshape(4, 16)
    acc = np.zeros_like(x)
    n = 4000
    for s in range(n):
        y, f = O._drop(x, dict(p=0.25, seed=11, stream=s), 2)
        assert set(np.unique(f)) <= {0.0, 1.0 / 0.75}
        acc += y
    assert np.allclose(acc / n, x, atol=6 * 3.0 * math.sqrt(0.25 / 0.75 / n))
    y0, f0 = O._drop(x, dict(p=0.0, seed=11, stream=0), 2)
    assert y0 is x and f0 is None
    cfg = MICRO
    th = micro_theta(cfg, 5)
    mb = micro_batch(cfg, [8, 4], 8, 3)
    a = O.micro_batch_grad(cfg, th, mb["ids"], mb["lens"], mb["mlm_pos"], mb["mlm_label"])
    b = O.micro_batch_grad(cfg, th, mb["ids"], mb["lens"], mb["mlm_pos"], mb["mlm_label"], dict(p=0.0, seed=1, stream=1))
    assert a[0] == b[0] and np.array_equal(a[1], b[1])


def test_gradients_with_dropout_match_finite_differences_fp64():
    """With the masks fixed by (seed, stream) the dropped network is an ordinary differentiable
    function: central differences pin the backward pass through all four kinds of sites."""
    cfg = MICRO
    th = micro_theta(cfg, 31)
    mb = micro_batch(cfg, [8, 3, 5], 8, 19)
    drop = dict(p=0.3, seed=99, stream=7)

    def loss_d(theta):
        hidden, _ = O.encoder_forward(cfg, theta, mb["ids"], mb["lens"], drop)
        return float(O.mlm_loss_forward(cfg, theta, hidden, mb["mlm_pos"], mb["mlm_label"])[0])

    loss, grad, _, _ = O.micro_batch_grad(cfg, th, mb["ids"], mb["lens"], mb["mlm_pos"], mb["mlm_label"], drop)
    assert loss == pytest.approx(loss_d(th), rel=1e-14)
    assert abs(loss - loss_of(cfg, th, mb)) > 1e-3          # dropout did change the function
    rng = np.random.default_rng(8)
    eps = 1e-5
    for name, off, r, c in O.param_layout(cfg):
        n = r * c
        u = np.zeros_like(th)
        u[off:off + n] = rng.standard_normal(n)
        fd = (loss_d(th + eps * u) - loss_d(th - eps * u)) / (2 * eps)
        an = float(grad @ u)
        assert abs(fd - an) <= 1e-6 * max(abs(fd), abs(an)) + 1e-9, (name, fd, an)
