"""Plain NumPy oracle of one worker's share of a HetSeq training step.

TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct definition that
the HIP kernels are compared with.  It is never part of the product path, shares no
code with it and does not import it.

What the paper (HetSeq, "Distributed GPU Training on Heterogeneous Infrastructure")
fixes, and where:

* Section "Optimizer and Learning Rate Scheduler": workers run unequal batches, so
  every worker reports its loss together with a weight (batch size or token count)
  and the weighted sum over workers, divided by the total weight, is what is
  trained on.  Here: each micro-batch returns a loss SUM, gradients of the sums are
  added, and the total is divided by the global sample count (`normalize`).
* Section "Backpropagation": a worker without data runs a dummy batch whose gradient
  is set to zero, i.e. it contributes nothing (`accumulate(..., ignore=True)`).
* Section "Delayed Update (Gradient Accumulation)": several forward/backward passes
  are aggregated before one update and the batch size scales with their number
  (`accumulate` called once per micro-batch, sample counts added).
* Section "Forward Pass": batches are formed under a max-instances or max-tokens
  criterion (see `oracle/batcher.py`).
* Section "BERT Language Model": Adam with beta1 0.9, beta2 0.999, eps 1e-8,
  maximum learning rate 1e-4 (`adam_step`); linear-decay schedule with 10K warm-up updates of
  1M (`lr_linear`).
* Section "Transformer Translation Model" trains with dropout 0.1 and section "Checkpointing" keeps
  the random seed in the snapshot; the cited BERT model drops, with the same rate, its embedding
  output, attention probabilities, attention output and feed-forward output.  `encoder_forward(...,
  drop)` does so with a counter-based generator, so that a mask is a pure function of (seed,
  stream, site, element) and both sides of a comparison can produce it.
* Section "Checkpointing": a snapshot holds the parameters, the completed steps, the optimizer
  status with the scheduler's and the seed; training continues from it exactly (`train_loop`
  works on such a state).

The transformer encoder itself is only cited by the paper (BERT); the textbook
definition is written out below: post-LN encoder layers, softmax attention that
excludes padded keys, exact-erf GELU, LayerNorm with biased variance, a masked-LM
head whose decoder is tied to the word embedding, cross-entropy summed over targets.

Precision is a parameter (`dtype`): float32 is the reference precision, float64 is
used for finite-difference checks and as a tighter reference on small cases.

Pins (tests/test_oracle_*.py): central finite differences in float64 for every
parameter tensor; a pure-Python loop re-implementation of the forward pass; SciPy's
logsumexp/erf; padding invariance; the concatenation invariant
sum_i grad_i / sum_i n_i == grad(concatenated batch)/D; the paper's worked example
with local batch sizes 2,2,1,0; Adam closed forms; the schedule's closed-form values at the
paper's settings; a loop interrupted and resumed equals the uninterrupted one bit for bit;
the generator's published known-answer vectors, mask frequency and independence, unbiasedness,
and finite differences through all four kinds of dropout sites.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np
from scipy.special import erf

PAD_ID = 0
MASK_ID = 4


@dataclass(frozen=True)
class ModelCfg:
    n_layers: int
    hidden: int
    n_heads: int
    ffn: int
    vocab: int
    max_pos: int
    ln_eps: float = 1e-12

    @property
    def head_dim(self) -> int:
        return self.hidden // self.n_heads


# --------------------------------------------------------------------------------------
# flat parameter layout (the oracle's own statement of it; the HIP library has its own,
# and a test checks that the two agree)
# --------------------------------------------------------------------------------------
def param_layout(cfg: ModelCfg):
    """List of (name, offset, rows, cols); vectors have rows == 1.  Weights are
    [out, in] row-major (y = x W^T + b)."""
    H, F, V = cfg.hidden, cfg.ffn, cfg.vocab
    shapes = [("emb.word", V, H), ("emb.pos", cfg.max_pos, H), ("emb.ln.g", 1, H), ("emb.ln.b", 1, H)]
    for i in range(cfg.n_layers):
        p = f"l{i}."
        shapes += [
            (p + "qkv.w", 3 * H, H), (p + "qkv.b", 1, 3 * H),
            (p + "o.w", H, H), (p + "o.b", 1, H),
            (p + "ln1.g", 1, H), (p + "ln1.b", 1, H),
            (p + "ffn1.w", F, H), (p + "ffn1.b", 1, F),
            (p + "ffn2.w", H, F), (p + "ffn2.b", 1, H),
            (p + "ln2.g", 1, H), (p + "ln2.b", 1, H),
        ]
    shapes += [("head.t.w", H, H), ("head.t.b", 1, H), ("head.ln.g", 1, H), ("head.ln.b", 1, H),
               ("head.dec.b", 1, V)]
    out, off = [], 0
    for name, r, c in shapes:
        out.append((name, off, r, c))
        off += r * c
    return out


def param_count(cfg: ModelCfg) -> int:
    name, off, r, c = param_layout(cfg)[-1]
    return off + r * c


def param_views(cfg: ModelCfg, flat: np.ndarray) -> dict:
    """Named views into a flat parameter (or gradient) vector; vectors are 1-D."""
    assert flat.ndim == 1 and flat.size == param_count(cfg)
    views = {}
    for name, off, r, c in param_layout(cfg):
        v = flat[off:off + r * c]
        views[name] = v if r == 1 else v.reshape(r, c)
    return views


# --------------------------------------------------------------------------------------
# building blocks
# --------------------------------------------------------------------------------------
def key_mask(lens: np.ndarray, L: int) -> np.ndarray:
    """mask[b, l] = 1 where position l of sequence b is a real token."""
    return (np.arange(L)[None, :] < np.asarray(lens)[:, None]).astype(np.uint8)


def gelu(x):
    return 0.5 * x * (1.0 + erf(x / math.sqrt(2.0)))


def gelu_grad(x):
    return 0.5 * (1.0 + erf(x / math.sqrt(2.0))) + x * np.exp(-0.5 * x * x) / math.sqrt(2.0 * math.pi)


def layer_norm_fwd(x, gain, bias, eps):
    """y = (x - mean) / sqrt(var + eps) * gain + bias, biased variance over the last axis."""
    mu = x.mean(axis=-1, keepdims=True)
    xc = x - mu
    var = (xc * xc).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + x.dtype.type(eps))
    xhat = xc * rstd
    return xhat * gain + bias, (xhat, rstd)


def layer_norm_bwd(dy, cache, gain):
    xhat, rstd = cache
    H = dy.shape[-1]
    d_gain = (dy * xhat).reshape(-1, H).sum(axis=0)
    d_bias = dy.reshape(-1, H).sum(axis=0)
    dxhat = dy * gain
    dx = rstd * (dxhat - dxhat.mean(axis=-1, keepdims=True)
                 - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True))
    return dx, d_gain, d_bias


# --------------------------------------------------------------------------------------
# dropout with a counter-based generator
# --------------------------------------------------------------------------------------
# The generator is Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random numbers:
# as easy as 1, 2, 3", SC'11), written from its published definition: a 4 x 32-bit counter and a
# 2 x 32-bit key go through 10 rounds; a round replaces (c0, c1, c2, c3) by
# (hi(M1*c2) ^ c1 ^ k0, lo(M1*c2), hi(M0*c0) ^ c3 ^ k1, lo(M0*c0)) and the key is bumped by the two
# Weyl constants between rounds.
PHILOX_M0, PHILOX_M1 = 0xD2511F53, 0xCD9E8D57
PHILOX_W0, PHILOX_W1 = 0x9E3779B9, 0xBB67AE85


def philox4x32_10(counter: np.ndarray, key) -> np.ndarray:
    """counter: uint32 [..., 4]; key: two 32-bit integers.  Returns uint32 [..., 4]."""
    c = [counter[..., j].astype(np.uint64) for j in range(4)]
    k0, k1 = np.uint64(key[0] & 0xFFFFFFFF), np.uint64(key[1] & 0xFFFFFFFF)
    mask = np.uint64(0xFFFFFFFF)
    for _ in range(10):
        p0 = np.uint64(PHILOX_M0) * c[0]
        p1 = np.uint64(PHILOX_M1) * c[2]
        c = [(p1 >> np.uint64(32)) ^ c[1] ^ k0, p1 & mask, (p0 >> np.uint64(32)) ^ c[3] ^ k1, p0 & mask]
        k0 = (k0 + np.uint64(PHILOX_W0)) & mask
        k1 = (k1 + np.uint64(PHILOX_W1)) & mask
    return np.stack(c, axis=-1).astype(np.uint32)


def dropout_keep(drop: dict, site: int, n: int) -> np.ndarray:
    """Which of the n elements of dropout site `site` survive.  Element e uses word e % 4 of the block
    with counter (e // 4 low, e // 4 high, site, drop['stream']) under the key (seed low, seed high);
    it is dropped when that word is below floor(p * 2^32).  `stream` tells apart the micro-batches
    and updates of a run; the seed is the run's (section "Checkpointing" keeps it in the snapshot)."""
    groups = (n + 3) // 4
    g = np.arange(groups, dtype=np.uint64)
    counter = np.empty((groups, 4), dtype=np.uint32)
    counter[:, 0] = (g & np.uint64(0xFFFFFFFF)).astype(np.uint32)
    counter[:, 1] = (g >> np.uint64(32)).astype(np.uint32)
    counter[:, 2] = np.uint32(site)
    counter[:, 3] = np.uint32(drop["stream"] & 0xFFFFFFFF)
    seed = int(drop["seed"])
    words = philox4x32_10(counter, (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)).reshape(-1)[:n]
    thr = np.uint32(min(int(math.floor(drop["p"] * 4294967296.0)), 0xFFFFFFFF))
    return words >= thr


def _drop(x: np.ndarray, drop, site: int):
    """Inverted dropout: survivors are scaled by 1 / (1 - p).  Returns (y, factor) with y = x * factor."""
    if drop is None or drop["p"] <= 0.0:
        return x, None
    keep = dropout_keep(drop, site, x.size).reshape(x.shape)
    factor = keep.astype(x.dtype) * x.dtype.type(1.0 / (1.0 - drop["p"]))
    return x * factor, factor


def site_embedding() -> int:
    return 0


def site_attention_prob(layer: int) -> int:
    return 1 + 3 * layer


def site_attention_out(layer: int) -> int:
    return 2 + 3 * layer


def site_ffn_out(layer: int) -> int:
    return 3 + 3 * layer


# --------------------------------------------------------------------------------------
# forward: encoder, then masked-LM head and loss SUM
# --------------------------------------------------------------------------------------
def encoder_forward(cfg: ModelCfg, theta: np.ndarray, ids: np.ndarray, lens: np.ndarray, drop=None):
    """ids [B, L] int, lens [B] (each >= 1).  Returns hidden [B, L, H] and a cache.
    drop = dict(p, seed, stream) switches on dropout at BERT's four kinds of sites: the embedding
    output, the attention probabilities, the attention output and the feed-forward output (the last
    two before the residual is added)."""
    P = param_views(cfg, theta)
    dt = theta.dtype
    B, L = ids.shape
    H, A, d = cfg.hidden, cfg.n_heads, cfg.head_dim
    assert L <= cfg.max_pos and np.all(np.asarray(lens) >= 1) and np.all(np.asarray(lens) <= L)
    valid = key_mask(lens, L).astype(bool)                       # [B, L]

    e = P["emb.word"][ids] + P["emb.pos"][:L][None, :, :]
    x, c_emb = layer_norm_fwd(e, P["emb.ln.g"], P["emb.ln.b"], cfg.ln_eps)
    x, f_emb = _drop(x, drop, site_embedding())
    cache = {"ids": ids, "lens": np.asarray(lens), "valid": valid, "emb_ln": c_emb, "f_emb": f_emb, "layers": []}
    scale = dt.type(1.0 / math.sqrt(d))
    for i in range(cfg.n_layers):
        p = f"l{i}."
        qkv = x @ P[p + "qkv.w"].T + P[p + "qkv.b"]              # [B, L, 3H]
        q, k, v = (qkv[..., j * H:(j + 1) * H].reshape(B, L, A, d).transpose(0, 2, 1, 3) for j in range(3))
        s = (q @ k.transpose(0, 1, 3, 2)) * scale                # [B, A, L, L]
        s = np.where(valid[:, None, None, :], s, -np.inf)       # padded keys are excluded
        s_max = s.max(axis=-1, keepdims=True)
        pexp = np.exp(s - s_max)
        prob = pexp / pexp.sum(axis=-1, keepdims=True)
        probd, f_prob = _drop(prob, drop, site_attention_prob(i))
        ctx = (probd @ v).transpose(0, 2, 1, 3).reshape(B, L, H)
        ao, f_ao = _drop(ctx @ P[p + "o.w"].T + P[p + "o.b"], drop, site_attention_out(i))
        y1 = x + ao
        x1, c_ln1 = layer_norm_fwd(y1, P[p + "ln1.g"], P[p + "ln1.b"], cfg.ln_eps)
        hpre = x1 @ P[p + "ffn1.w"].T + P[p + "ffn1.b"]
        h = gelu(hpre)
        fo, f_fo = _drop(h @ P[p + "ffn2.w"].T + P[p + "ffn2.b"], drop, site_ffn_out(i))
        y2 = x1 + fo
        x2, c_ln2 = layer_norm_fwd(y2, P[p + "ln2.g"], P[p + "ln2.b"], cfg.ln_eps)
        cache["layers"].append(dict(x=x, q=q, k=k, v=v, prob=prob, probd=probd, ctx=ctx, ln1=c_ln1, x1=x1,
                                    hpre=hpre, h=h, ln2=c_ln2, f_prob=f_prob, f_ao=f_ao, f_fo=f_fo))
        x = x2
    return x, cache


def mlm_loss_forward(cfg: ModelCfg, theta: np.ndarray, hidden: np.ndarray, mlm_pos, mlm_label):
    """loss_sum = sum_m [logsumexp(logits_m) - logits_m[label_m]]; no division here: the
    weight (sample or token count) travels beside the sum."""
    P = param_views(cfg, theta)
    H = cfg.hidden
    mlm_pos = np.asarray(mlm_pos, dtype=np.int64)
    mlm_label = np.asarray(mlm_label, dtype=np.int64)
    g = hidden.reshape(-1, H)[mlm_pos]                          # [M, H]
    tpre = g @ P["head.t.w"].T + P["head.t.b"]
    tact = gelu(tpre)
    t, c_ln = layer_norm_fwd(tact, P["head.ln.g"], P["head.ln.b"], cfg.ln_eps)
    logits = t @ P["emb.word"].T + P["head.dec.b"]              # tied decoder
    M = logits.shape[0]
    if M == 0:
        return theta.dtype.type(0.0), dict(M=0, mlm_pos=mlm_pos)
    zmax = logits.max(axis=1, keepdims=True)
    lse = zmax[:, 0] + np.log(np.exp(logits - zmax).sum(axis=1))
    loss_sum = (lse - logits[np.arange(M), mlm_label]).sum()
    cache = dict(M=M, mlm_pos=mlm_pos, mlm_label=mlm_label, g=g, tpre=tpre, tact=tact, t=t, ln=c_ln,
                 logits=logits, lse=lse)
    return loss_sum, cache


# --------------------------------------------------------------------------------------
# backward
# --------------------------------------------------------------------------------------
def mlm_loss_backward(cfg: ModelCfg, theta: np.ndarray, hidden_shape, cache, grad: np.ndarray):
    """Adds the head's parameter gradients (and the decoder part of the tied word
    embedding) into `grad`; returns d loss_sum / d hidden (zero off the target rows)."""
    P = param_views(cfg, theta)
    G = param_views(cfg, grad)
    d_hidden = np.zeros(hidden_shape, dtype=theta.dtype)
    M = cache["M"]
    if M == 0:
        return d_hidden
    dlogits = np.exp(cache["logits"] - cache["lse"][:, None])    # softmax
    dlogits[np.arange(M), cache["mlm_label"]] -= 1.0
    G["head.dec.b"] += dlogits.sum(axis=0)
    G["emb.word"] += dlogits.T @ cache["t"]
    dt_ = dlogits @ P["emb.word"]
    dtact, dg_, db_ = layer_norm_bwd(dt_, cache["ln"], P["head.ln.g"])
    G["head.ln.g"] += dg_
    G["head.ln.b"] += db_
    dtpre = dtact * gelu_grad(cache["tpre"])
    G["head.t.w"] += dtpre.T @ cache["g"]
    G["head.t.b"] += dtpre.sum(axis=0)
    dgath = dtpre @ P["head.t.w"]
    flat = d_hidden.reshape(-1, cfg.hidden)
    np.add.at(flat, cache["mlm_pos"], dgath)
    return d_hidden


def encoder_backward(cfg: ModelCfg, theta: np.ndarray, cache, d_hidden: np.ndarray, grad: np.ndarray):
    """Chain rule through the encoder; parameter gradients are added into `grad`."""
    P = param_views(cfg, theta)
    G = param_views(cfg, grad)
    dt = theta.dtype
    H, A, d = cfg.hidden, cfg.n_heads, cfg.head_dim
    B, L = cache["ids"].shape
    T = B * L
    scale = dt.type(1.0 / math.sqrt(d))
    dx = d_hidden
    for i in reversed(range(cfg.n_layers)):
        p = f"l{i}."
        c = cache["layers"][i]
        dy2, dg_, db_ = layer_norm_bwd(dx, c["ln2"], P[p + "ln2.g"])
        G[p + "ln2.g"] += dg_
        G[p + "ln2.b"] += db_
        dfo = dy2 if c["f_fo"] is None else dy2 * c["f_fo"]        # through the dropout of the FFN output
        dy2f = dfo.reshape(T, H)
        G[p + "ffn2.b"] += dy2f.sum(axis=0)
        G[p + "ffn2.w"] += dy2f.T @ c["h"].reshape(T, -1)
        dh = dfo @ P[p + "ffn2.w"]
        dhpre = dh * gelu_grad(c["hpre"])
        dhpf = dhpre.reshape(T, -1)
        G[p + "ffn1.b"] += dhpf.sum(axis=0)
        G[p + "ffn1.w"] += dhpf.T @ c["x1"].reshape(T, H)
        dx1 = dy2 + dhpre @ P[p + "ffn1.w"]
        dy1, dg_, db_ = layer_norm_bwd(dx1, c["ln1"], P[p + "ln1.g"])
        G[p + "ln1.g"] += dg_
        G[p + "ln1.b"] += db_
        dao = dy1 if c["f_ao"] is None else dy1 * c["f_ao"]        # through the dropout of the attention output
        dy1f = dao.reshape(T, H)
        G[p + "o.b"] += dy1f.sum(axis=0)
        G[p + "o.w"] += dy1f.T @ c["ctx"].reshape(T, H)
        dctx = (dao @ P[p + "o.w"]).reshape(B, L, A, d).transpose(0, 2, 1, 3)     # [B, A, L, d]
        prob, q, k, v = c["prob"], c["q"], c["k"], c["v"]
        dv = c["probd"].transpose(0, 1, 3, 2) @ dctx
        dprob = dctx @ v.transpose(0, 1, 3, 2)
        if c["f_prob"] is not None:
            dprob = dprob * c["f_prob"]                           # through the dropout of the probabilities
        ds = prob * (dprob - (dprob * prob).sum(axis=-1, keepdims=True))          # softmax backward
        dq = (ds @ k) * scale
        dk = (ds.transpose(0, 1, 3, 2) @ q) * scale
        dqkv = np.concatenate([a.transpose(0, 2, 1, 3).reshape(B, L, H) for a in (dq, dk, dv)], axis=-1)
        dqkvf = dqkv.reshape(T, 3 * H)
        G[p + "qkv.b"] += dqkvf.sum(axis=0)
        G[p + "qkv.w"] += dqkvf.T @ c["x"].reshape(T, H)
        dx = dy1 + dqkv @ P[p + "qkv.w"]
    if cache["f_emb"] is not None:
        dx = dx * cache["f_emb"]
    de, dg_, db_ = layer_norm_bwd(dx, cache["emb_ln"], P["emb.ln.g"])
    G["emb.ln.g"] += dg_
    G["emb.ln.b"] += db_
    G["emb.pos"][:L] += de.sum(axis=0)
    np.add.at(G["emb.word"], cache["ids"].reshape(-1), de.reshape(T, H))          # duplicates summed


def micro_batch_grad(cfg: ModelCfg, theta: np.ndarray, ids, lens, mlm_pos, mlm_label, drop=None):
    """One forward/backward pass of one micro-batch.  Returns (loss_sum, flat gradient of
    loss_sum, n_seq, n_tok)."""
    ids = np.asarray(ids)
    hidden, cache = encoder_forward(cfg, theta, ids, lens, drop)
    loss_sum, hcache = mlm_loss_forward(cfg, theta, hidden, mlm_pos, mlm_label)
    grad = np.zeros_like(theta)
    d_hidden = mlm_loss_backward(cfg, theta, hidden.shape, hcache, grad)
    encoder_backward(cfg, theta, cache, d_hidden, grad)
    return loss_sum, grad, ids.shape[0], int(hcache["M"])


# --------------------------------------------------------------------------------------
# accumulate, normalise, Adam
# --------------------------------------------------------------------------------------
def accumulate(G: np.ndarray, n_total, g, n, ignore: bool = False):
    """Delayed update: G += g, n_total += n.  A dummy micro-batch (ignore) contributes
    neither; its gradient is not even read."""
    if ignore:
        return G, n_total
    G += g
    return G, n_total + n


def normalize(G: np.ndarray, denom):
    """G <- G / D with D the global weight (sample count summed over all micro-batches
    and workers)."""
    assert denom > 0
    G /= G.dtype.type(denom)
    return G


def adam_step(w, m, v, G, t: int, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0):
    """Adam with bias correction, eps added to sqrt(v_hat); t is 1-based.  Weight decay,
    when non-zero, is decoupled: w <- w - lr * wd * w.  Updates in place."""
    assert t >= 1
    ty = w.dtype.type
    m *= ty(beta1)
    m += ty(1.0 - beta1) * G
    v *= ty(beta2)
    v += ty(1.0 - beta2) * (G * G)
    mhat = m / ty(1.0 - beta1 ** t)
    vhat = v / ty(1.0 - beta2 ** t)
    if weight_decay != 0.0:
        w -= ty(lr * weight_decay) * w
    w -= ty(lr) * mhat / (np.sqrt(vhat) + ty(eps))
    return w, m, v


def train_step(cfg: ModelCfg, theta, m, v, t, micro_batches, lr=1e-4, beta1=0.9, beta2=0.999,
               eps=1e-8, weight_decay=0.0, denom=None):
    """The whole hot path.  micro_batches: list of dicts with ids, lens, mlm_pos,
    mlm_label and optionally dummy=True.  Returns (reported loss = sum of loss sums / D,
    normalised gradient G, D).  theta, m, v are updated in place."""
    G = np.zeros_like(theta)
    n_total, loss_total = 0, 0.0
    for mb in micro_batches:
        if mb.get("dummy", False):
            G, n_total = accumulate(G, n_total, None, 0, ignore=True)
            continue
        loss_sum, g, n_seq, _ = micro_batch_grad(cfg, theta, mb["ids"], mb["lens"], mb["mlm_pos"], mb["mlm_label"],
                                                 mb.get("drop"))
        G, n_total = accumulate(G, n_total, g, n_seq)
        loss_total += float(loss_sum)
    D = n_total if denom is None else denom
    normalize(G, D)
    adam_step(theta, m, v, G, t, lr, beta1, beta2, eps, weight_decay)
    return loss_total / D, G, D


# ----------------------------------------------------------------------------------------------
# Training loop: learning-rate schedule and resumable state
# ----------------------------------------------------------------------------------------------
def lr_linear(t: int, max_lr: float, warmup: int, total: int) -> float:
    """Learning rate of update number t = 1, 2, ... under the linear schedule of section "BERT
    Language Model" (linear decay, maximum rate, the first `warmup` updates as warm-up, `total`
    updates in all).  The paper gives the three numbers only; the usual reading is taken: the rate
    rises linearly from 0 to max_lr over the warm-up (max_lr * t / warmup, reaching max_lr at
    t = warmup) and then falls linearly to 0 at t = total; it is 0 beyond."""
    if t < 1 or warmup < 0 or total < max(warmup, 1):
        raise ValueError("lr_linear: need t >= 1 and 0 <= warmup <= total")
    if t <= warmup:
        return max_lr * t / warmup
    if t >= total:
        return 0.0
    return max_lr * (total - t) / (total - warmup)


def train_loop(cfg: ModelCfg, state: dict, n_steps: int, micro_batches_of, adam: dict, schedule: dict):
    """n_steps updates from `state` = dict(theta, m, v, step) (updated in place; `step` counts the
    completed updates, which is what section "Checkpointing" stores next to the parameters, the
    optimizer status and the seed).  Update number t = step + 1 takes its micro-batches from
    micro_batches_of(t) and its rate from lr_linear(t, **schedule).  Returns the reported losses."""
    losses = []
    for _ in range(n_steps):
        t = state["step"] + 1
        lr = lr_linear(t, schedule["max_lr"], schedule["warmup"], schedule["total"])
        loss, _, _ = train_step(cfg, state["theta"], state["m"], state["v"], t, micro_batches_of(t), lr=lr,
                                beta1=adam["beta1"], beta2=adam["beta2"], eps=adam["eps"],
                                weight_decay=adam.get("weight_decay", 0.0))
        state["step"] = t
        losses.append(loss)
    return losses
