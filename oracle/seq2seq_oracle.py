"""Plain NumPy oracle of one worker's share of a training step of the translation workload.

TEST INFRASTRUCTURE ONLY.  Slow, obviously-correct definition that the HIP path is compared
with; never part of the product path, shares no code with it and does not import it.

What the paper fixes (section "Transformer Translation Model"): the base Transformer of
Vaswani et al. ("Attention is all you need") with 6 encoder and 6 decoder layers, hidden size
512, 8 heads, dropout 0.1, label-smoothed cross-entropy with epsilon 0.1, about 65 million
parameters, Adam with beta1 0.9, beta2 0.98, eps 1e-9; Table 1 trains it with 4096 tokens per
GPU.  The model itself is only cited, so the published definition is written out here:

* one embedding matrix shared by source tokens, target tokens and the output projection;
  inputs are sqrt(H) * E[id] + PE[position] with the fixed sinusoidal table
  PE[p, 2i] = sin(p / 10000^(2i/H)), PE[p, 2i+1] = cos(p / 10000^(2i/H));
* post-LN sub-layers x <- LN(x + drop(sublayer(x))): encoder layers = self-attention, ReLU
  feed-forward; decoder layers = causal self-attention, attention over the encoder output
  (keys and values from the encoder, queries from the decoder), ReLU feed-forward;
* dropout on the two embedding sums and on every sub-layer output (the cited paper's residual
  dropout), none on attention probabilities;
* logits = decoder output times E^T (no bias);
* label smoothing (Szegedy et al., "Rethinking the Inception architecture"): the target
  distribution of a token is (1 - eps) on its label plus eps / V on every class, and the loss
  is the cross-entropy to it, summed over the real target tokens (no division here: the
  weight travels beside the sum, section "Optimizer and Learning Rate Scheduler").

Pins (tests/test_oracle_seq2seq.py): central finite differences in float64 for every parameter
tensor, with and without dropout; a pure-Python loop re-implementation of masked attention;
causality (an output position does not see later target tokens); padding invariance on both
sides; label smoothing against -sum q log p written out, its eps = 0 and uniform-logit closed
forms; closed-form entries of the positional table; one-key attention; the parameter count of
the base model against the paper's "about 65 million".
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

from .hetseq_oracle import _drop, layer_norm_bwd, layer_norm_fwd

PAD_ID = 0


@dataclass(frozen=True)
class S2SCfg:
    n_enc: int
    n_dec: int
    hidden: int
    n_heads: int
    ffn: int
    vocab: int
    max_pos: int
    ln_eps: float = 1e-5

    @property
    def head_dim(self) -> int:
        return self.hidden // self.n_heads


# --------------------------------------------------------------------------------------
# flat parameter buffer
# --------------------------------------------------------------------------------------
def param_layout(cfg: S2SCfg):
    """(name, offset, rows, cols) in buffer order; weights are [out, in], vectors [1, n]."""
    H, F, V = cfg.hidden, cfg.ffn, cfg.vocab
    out, off = [], 0

    def add(name, r, c):
        nonlocal off
        out.append((name, off, r, c))
        off += r * c

    def attn_ffn(p, cross):
        add(p + "qkv.w", 3 * H, H); add(p + "qkv.b", 1, 3 * H)
        add(p + "o.w", H, H); add(p + "o.b", 1, H)
        add(p + "ln1.g", 1, H); add(p + "ln1.b", 1, H)
        if cross:
            add(p + "cq.w", H, H); add(p + "cq.b", 1, H)
            add(p + "ckv.w", 2 * H, H); add(p + "ckv.b", 1, 2 * H)
            add(p + "co.w", H, H); add(p + "co.b", 1, H)
            add(p + "lnc.g", 1, H); add(p + "lnc.b", 1, H)
        add(p + "ffn1.w", F, H); add(p + "ffn1.b", 1, F)
        add(p + "ffn2.w", H, F); add(p + "ffn2.b", 1, H)
        add(p + "ln2.g", 1, H); add(p + "ln2.b", 1, H)

    add("emb", V, H)
    for i in range(cfg.n_enc):
        attn_ffn(f"enc{i}.", False)
    for i in range(cfg.n_dec):
        attn_ffn(f"dec{i}.", True)
    return out


def param_count(cfg: S2SCfg) -> int:
    name, off, r, c = param_layout(cfg)[-1]
    return off + r * c


def param_views(cfg: S2SCfg, flat: np.ndarray) -> dict:
    return {name: flat[off:off + r * c].reshape(r, c) if r > 1 else flat[off:off + c]
            for name, off, r, c in param_layout(cfg)}


def positional_table(n_pos: int, H: int, dtype=np.float64) -> np.ndarray:
    """PE[p, 2i] = sin(p / 10000^(2i/H)), PE[p, 2i+1] = cos(p / 10000^(2i/H)), evaluated in float64."""
    p = np.arange(n_pos, dtype=np.float64)[:, None]
    i = np.arange(H // 2, dtype=np.float64)[None, :]
    angle = p / np.power(10000.0, 2.0 * i / H)
    pe = np.empty((n_pos, H), dtype=np.float64)
    pe[:, 0::2] = np.sin(angle)
    pe[:, 1::2] = np.cos(angle)
    return pe.astype(dtype)


# --------------------------------------------------------------------------------------
# dropout sites (element index = row-major index of the tensor the mask applies to)
# --------------------------------------------------------------------------------------
def site_src_embedding() -> int:
    return 0


def site_tgt_embedding() -> int:
    return 1


def site_enc(layer: int, which: int) -> int:
    """which: 0 attention output, 1 feed-forward output."""
    return 2 + 2 * layer + which


def site_dec(cfg: S2SCfg, layer: int, which: int) -> int:
    """which: 0 self-attention output, 1 encoder-attention output, 2 feed-forward output."""
    return 2 + 2 * cfg.n_enc + 3 * layer + which


# --------------------------------------------------------------------------------------
# multi-head attention with an explicit table of allowed (query, key) pairs
# --------------------------------------------------------------------------------------
def attention_forward(q, k, v, allowed, A):
    """q [B, Lq, H], k, v [B, Lk, H], allowed [B, Lq, Lk] bool (every query has at least one allowed
    key).  Returns ctx [B, Lq, H] and the cache for the backward pass."""
    B, Lq, H = q.shape
    Lk = k.shape[1]
    d = H // A
    qh = q.reshape(B, Lq, A, d).transpose(0, 2, 1, 3)
    kh = k.reshape(B, Lk, A, d).transpose(0, 2, 1, 3)
    vh = v.reshape(B, Lk, A, d).transpose(0, 2, 1, 3)
    s = (qh @ kh.transpose(0, 1, 3, 2)) * q.dtype.type(1.0 / math.sqrt(d))
    s = np.where(allowed[:, None, :, :], s, -np.inf)
    e = np.exp(s - s.max(axis=-1, keepdims=True))
    prob = e / e.sum(axis=-1, keepdims=True)
    ctx = (prob @ vh).transpose(0, 2, 1, 3).reshape(B, Lq, H)
    return ctx, (qh, kh, vh, prob)


def attention_backward(dctx, cache, A):
    """Returns dq [B, Lq, H], dk, dv [B, Lk, H]."""
    qh, kh, vh, prob = cache
    B, _, Lq, d = qh.shape
    Lk = kh.shape[2]
    H = A * d
    dch = dctx.reshape(B, Lq, A, d).transpose(0, 2, 1, 3)
    dv = prob.transpose(0, 1, 3, 2) @ dch
    dprob = dch @ vh.transpose(0, 1, 3, 2)
    ds = prob * (dprob - (dprob * prob).sum(axis=-1, keepdims=True))
    scale = dctx.dtype.type(1.0 / math.sqrt(d))
    dq = (ds @ kh) * scale
    dk = (ds.transpose(0, 1, 3, 2) @ qh) * scale
    back = lambda t, L: t.transpose(0, 2, 1, 3).reshape(B, L, H)
    return back(dq, Lq), back(dk, Lk), back(dv, Lk)


def allowed_pairs(q_len_padded: int, k_lens, k_len_padded: int, causal: bool) -> np.ndarray:
    """allowed[b, i, j]: key j is a real token of sequence b and, if causal, j <= i."""
    ok = (np.arange(k_len_padded)[None, None, :] < np.asarray(k_lens)[:, None, None])
    ok = np.broadcast_to(ok, (len(k_lens), q_len_padded, k_len_padded)).copy()
    if causal:
        ok &= (np.arange(k_len_padded)[None, None, :] <= np.arange(q_len_padded)[None, :, None])
    return ok


# --------------------------------------------------------------------------------------
# forward
# --------------------------------------------------------------------------------------
def _embed(cfg, P, ids, drop, site):
    L = ids.shape[1]
    dt = P["emb"].dtype
    x = P["emb"][ids] * dt.type(math.sqrt(cfg.hidden)) + positional_table(L, cfg.hidden, dt)[None]
    return _drop(x, drop, site)


def _ffn_fwd(P, p, x):
    h = np.maximum(x @ P[p + "ffn1.w"].T + P[p + "ffn1.b"], 0)
    return h @ P[p + "ffn2.w"].T + P[p + "ffn2.b"], h


def forward(cfg: S2SCfg, theta, src, src_lens, tgt_in, tgt_lens, drop=None):
    """src [B, Ls], tgt_in [B, Lt] int; lens >= 1.  Returns the decoder output [B, Lt, H] and a cache."""
    P = param_views(cfg, theta)
    H, A = cfg.hidden, cfg.n_heads
    B, Ls = src.shape
    Lt = tgt_in.shape[1]
    assert max(Ls, Lt) <= cfg.max_pos
    assert np.all(np.asarray(src_lens) >= 1) and np.all(np.asarray(src_lens) <= Ls)
    assert np.all(np.asarray(tgt_lens) >= 1) and np.all(np.asarray(tgt_lens) <= Lt)
    ok_enc = allowed_pairs(Ls, src_lens, Ls, False)
    ok_self = allowed_pairs(Lt, tgt_lens, Lt, True)
    ok_cross = allowed_pairs(Lt, src_lens, Ls, False)
    cache = dict(src=src, tgt_in=tgt_in, enc=[], dec=[])

    x, cache["f_src"] = _embed(cfg, P, src, drop, site_src_embedding())
    for i in range(cfg.n_enc):
        p = f"enc{i}."
        qkv = x @ P[p + "qkv.w"].T + P[p + "qkv.b"]
        ctx, c_att = attention_forward(qkv[..., :H], qkv[..., H:2 * H], qkv[..., 2 * H:], ok_enc, A)
        ao, f_ao = _drop(ctx @ P[p + "o.w"].T + P[p + "o.b"], drop, site_enc(i, 0))
        x1, c_ln1 = layer_norm_fwd(x + ao, P[p + "ln1.g"], P[p + "ln1.b"], cfg.ln_eps)
        f, h = _ffn_fwd(P, p, x1)
        fo, f_fo = _drop(f, drop, site_enc(i, 1))
        x2, c_ln2 = layer_norm_fwd(x1 + fo, P[p + "ln2.g"], P[p + "ln2.b"], cfg.ln_eps)
        cache["enc"].append(dict(x=x, att=c_att, ctx=ctx, f_ao=f_ao, ln1=c_ln1, x1=x1, h=h, f_fo=f_fo, ln2=c_ln2))
        x = x2
    enc_out = x

    y, cache["f_tgt"] = _embed(cfg, P, tgt_in, drop, site_tgt_embedding())
    for i in range(cfg.n_dec):
        p = f"dec{i}."
        qkv = y @ P[p + "qkv.w"].T + P[p + "qkv.b"]
        ctx, c_att = attention_forward(qkv[..., :H], qkv[..., H:2 * H], qkv[..., 2 * H:], ok_self, A)
        ao, f_ao = _drop(ctx @ P[p + "o.w"].T + P[p + "o.b"], drop, site_dec(cfg, i, 0))
        y1, c_ln1 = layer_norm_fwd(y + ao, P[p + "ln1.g"], P[p + "ln1.b"], cfg.ln_eps)
        cq = y1 @ P[p + "cq.w"].T + P[p + "cq.b"]
        ckv = enc_out @ P[p + "ckv.w"].T + P[p + "ckv.b"]
        cctx, c_catt = attention_forward(cq, ckv[..., :H], ckv[..., H:], ok_cross, A)
        co, f_co = _drop(cctx @ P[p + "co.w"].T + P[p + "co.b"], drop, site_dec(cfg, i, 1))
        yc, c_lnc = layer_norm_fwd(y1 + co, P[p + "lnc.g"], P[p + "lnc.b"], cfg.ln_eps)
        f, h = _ffn_fwd(P, p, yc)
        fo, f_fo = _drop(f, drop, site_dec(cfg, i, 2))
        y2, c_ln2 = layer_norm_fwd(yc + fo, P[p + "ln2.g"], P[p + "ln2.b"], cfg.ln_eps)
        cache["dec"].append(dict(y=y, att=c_att, ctx=ctx, f_ao=f_ao, ln1=c_ln1, y1=y1, catt=c_catt, cctx=cctx, f_co=f_co,
                                 lnc=c_lnc, yc=yc, h=h, f_fo=f_fo, ln2=c_ln2))
        y = y2
    cache["enc_out"] = enc_out
    return y, cache


def smoothed_ce(logits, labels, eps):
    """Rows with label < 0 are ignored.  Returns (loss_sum, nll_sum, d loss_sum / d logits).
    Per row: cross-entropy between q = (1 - eps) onehot(label) + eps / V and softmax(logits)."""
    labels = np.asarray(labels, dtype=np.int64)
    T, V = logits.shape
    use = labels >= 0
    zmax = logits.max(axis=1, keepdims=True)
    lse = zmax[:, 0] + np.log(np.exp(logits - zmax).sum(axis=1))
    lab = np.where(use, labels, 0)
    nll = lse - logits[np.arange(T), lab]
    smooth = lse - logits.mean(axis=1)          # = (1/V) sum_v (lse - z_v)
    dt = logits.dtype.type
    row = (dt(1.0) - dt(eps)) * nll + dt(eps) * smooth
    d = np.exp(logits - lse[:, None]) - dt(eps) / dt(V)
    d[np.arange(T), lab] -= dt(1.0) - dt(eps)
    d[~use] = 0
    return row[use].sum(), nll[use].sum(), d


def loss_forward_backward(cfg: S2SCfg, theta, dec_out, tgt_out, tgt_lens, eps, grad):
    """Output projection with the shared embedding and the smoothed loss over the real target tokens.
    Adds the projection's share of the embedding gradient into `grad`; returns (loss_sum, nll_sum,
    d loss_sum / d dec_out, n_tok)."""
    P = param_views(cfg, theta)
    G = param_views(cfg, grad)
    B, Lt, H = dec_out.shape
    real = np.arange(Lt)[None, :] < np.asarray(tgt_lens)[:, None]
    labels = np.where(real, tgt_out, -1).reshape(-1)
    t = dec_out.reshape(B * Lt, H)
    logits = t @ P["emb"].T
    loss_sum, nll_sum, dlogits = smoothed_ce(logits, labels, eps)
    G["emb"] += dlogits.T @ t
    return loss_sum, nll_sum, (dlogits @ P["emb"]).reshape(B, Lt, H), int(real.sum())


# --------------------------------------------------------------------------------------
# backward
# --------------------------------------------------------------------------------------
def _mask(d, f):
    return d if f is None else d * f


def _ffn_bwd(P, G, p, dfo, x_in, h, T):
    H = x_in.shape[-1]
    d2 = dfo.reshape(T, H)
    G[p + "ffn2.b"] += d2.sum(axis=0)
    G[p + "ffn2.w"] += d2.T @ h.reshape(T, -1)
    dh = (dfo @ P[p + "ffn2.w"]) * (h > 0)
    dhf = dh.reshape(T, -1)
    G[p + "ffn1.b"] += dhf.sum(axis=0)
    G[p + "ffn1.w"] += dhf.T @ x_in.reshape(T, H)
    return dh @ P[p + "ffn1.w"]


def _ln_bwd(P, G, name, dy, cache):
    dx, dg, db = layer_norm_bwd(dy, cache, P[name + ".g"])
    G[name + ".g"] += dg
    G[name + ".b"] += db
    return dx


def _self_attn_bwd(P, G, p, dao, c, x_in, A):
    B, L, H = x_in.shape
    T = B * L
    d1 = dao.reshape(T, H)
    G[p + "o.b"] += d1.sum(axis=0)
    G[p + "o.w"] += d1.T @ c["ctx"].reshape(T, H)
    dq, dk, dv = attention_backward(dao @ P[p + "o.w"], c["att"], A)
    dqkv = np.concatenate([dq, dk, dv], axis=-1).reshape(T, 3 * H)
    G[p + "qkv.b"] += dqkv.sum(axis=0)
    G[p + "qkv.w"] += dqkv.T @ x_in.reshape(T, H)
    return (dqkv @ P[p + "qkv.w"]).reshape(B, L, H)


def backward(cfg: S2SCfg, theta, cache, d_dec_out, grad):
    """Chain rule through decoder and encoder; parameter gradients are added into `grad`."""
    P = param_views(cfg, theta)
    G = param_views(cfg, grad)
    H, A = cfg.hidden, cfg.n_heads
    B, Lt = cache["tgt_in"].shape
    Ls = cache["src"].shape[1]
    Tt, Ts = B * Lt, B * Ls
    enc_out = cache["enc_out"]
    d_enc = np.zeros_like(enc_out)
    dy = d_dec_out
    for i in reversed(range(cfg.n_dec)):
        p = f"dec{i}."
        c = cache["dec"][i]
        dsum2 = _ln_bwd(P, G, p + "ln2", dy, c["ln2"])
        dyc = dsum2 + _ffn_bwd(P, G, p, _mask(dsum2, c["f_fo"]), c["yc"], c["h"], Tt)
        dsumc = _ln_bwd(P, G, p + "lnc", dyc, c["lnc"])
        dco = _mask(dsumc, c["f_co"])
        dcf = dco.reshape(Tt, H)
        G[p + "co.b"] += dcf.sum(axis=0)
        G[p + "co.w"] += dcf.T @ c["cctx"].reshape(Tt, H)
        dcq, dck, dcv = attention_backward(dco @ P[p + "co.w"], c["catt"], A)
        dckv = np.concatenate([dck, dcv], axis=-1).reshape(Ts, 2 * H)
        G[p + "ckv.b"] += dckv.sum(axis=0)
        G[p + "ckv.w"] += dckv.T @ enc_out.reshape(Ts, H)
        d_enc += (dckv @ P[p + "ckv.w"]).reshape(B, Ls, H)
        dcqf = dcq.reshape(Tt, H)
        G[p + "cq.b"] += dcqf.sum(axis=0)
        G[p + "cq.w"] += dcqf.T @ c["y1"].reshape(Tt, H)
        dy1 = dsumc + dcq @ P[p + "cq.w"]
        dsum1 = _ln_bwd(P, G, p + "ln1", dy1, c["ln1"])
        dy = dsum1 + _self_attn_bwd(P, G, p, _mask(dsum1, c["f_ao"]), c, c["y"], A)
    scale = theta.dtype.type(math.sqrt(H))
    np.add.at(G["emb"], cache["tgt_in"].reshape(-1), (_mask(dy, cache["f_tgt"]) * scale).reshape(Tt, H))

    dx = d_enc
    for i in reversed(range(cfg.n_enc)):
        p = f"enc{i}."
        c = cache["enc"][i]
        dsum2 = _ln_bwd(P, G, p + "ln2", dx, c["ln2"])
        dx1 = dsum2 + _ffn_bwd(P, G, p, _mask(dsum2, c["f_fo"]), c["x1"], c["h"], Ts)
        dsum1 = _ln_bwd(P, G, p + "ln1", dx1, c["ln1"])
        dx = dsum1 + _self_attn_bwd(P, G, p, _mask(dsum1, c["f_ao"]), c, c["x"], A)
    np.add.at(G["emb"], cache["src"].reshape(-1), (_mask(dx, cache["f_src"]) * scale).reshape(Ts, H))


def micro_batch_grad(cfg: S2SCfg, theta, mb: dict, eps: float = 0.1):
    """One forward/backward pass.  mb: src [B, Ls], src_lens, tgt_in [B, Lt], tgt_out [B, Lt], tgt_lens,
    optional drop = dict(p, seed, stream).  Returns (loss_sum, nll_sum, flat gradient of loss_sum,
    n_seq, n_tok) with n_tok the number of real target tokens."""
    dec_out, cache = forward(cfg, theta, mb["src"], mb["src_lens"], mb["tgt_in"], mb["tgt_lens"], mb.get("drop"))
    grad = np.zeros_like(theta)
    loss_sum, nll_sum, d_dec, n_tok = loss_forward_backward(cfg, theta, dec_out, mb["tgt_out"], mb["tgt_lens"], eps, grad)
    backward(cfg, theta, cache, d_dec, grad)
    return loss_sum, nll_sum, grad, mb["src"].shape[0], n_tok
