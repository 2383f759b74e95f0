"""Dropout on the GPU against the oracle: identical masks (both sides implement the same published
counter-based generator), then losses and gradients of whole micro-batches with dropout at all four
kinds of sites."""
import numpy as np
import pytest
import torch

from oracle import hetseq_oracle as O
from paper_2009_14783_amd import binding as hs
from paper_2009_14783_amd import synth
from paper_2009_14783_amd.step import Worker

pytestmark = pytest.mark.gpu


def rel(a, b):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    nb = np.linalg.norm(b)
    return np.linalg.norm(a - b) / nb if nb > 1e-12 else np.linalg.norm(a - b)


def test_keep_masks_are_bit_identical():
    cfg = hs.make_cfg(**synth.MODELS["tiny"], compute=hs.HS_FP32)
    ctx = hs.hs_ctx_create(cfg)
    for p, seed, stream, site, n in ((0.1, 0x0123456789ABCDEF, 7, 0, 100003), (0.5, 3, 0xFFFFFFFF, 22, 4096), (0.0, 1, 1, 1, 1000),
                                     (0.999, 2 ** 64 - 1, 5, 3, 70001)):
        hs.hs_set_dropout(ctx, p, seed, stream)
        got = torch.zeros(n, dtype=torch.uint8, device="cuda")
        hs.hs_dropout_keep_mask(ctx, site, n, got)
        torch.cuda.synchronize()
        want = O.dropout_keep(dict(p=p, seed=seed, stream=stream), site, n)
        assert np.array_equal(got.cpu().numpy().astype(bool), want), (p, seed, stream, site)
    with pytest.raises(hs.HsError):
        hs.hs_set_dropout(ctx, 1.0, 0, 0)
    with pytest.raises(hs.HsError):
        hs.hs_set_dropout(ctx, -0.1, 0, 0)
    hs.hs_ctx_destroy(ctx)


def run_case(model, compute, lens, L, drop, seed, tol, ids="uniform"):
    cfg = hs.make_cfg(**model)
    theta = synth.init_params(hs.hs_param_layout(cfg), seed)
    mb = synth.make_micro_batch(synth.rng_for(seed + 1), lens, L, model["vocab"], ids)
    ocfg = O.ModelCfg(**model)
    want_loss, want_g, _, _ = O.micro_batch_grad(ocfg, theta, mb["ids"], mb["lens"], mb["mlm_pos"], mb["mlm_label"], drop)
    plain_loss, plain_g, _, _ = O.micro_batch_grad(ocfg, theta, mb["ids"], mb["lens"], mb["mlm_pos"], mb["mlm_label"])
    wk = Worker(model, compute, theta)
    d = wk.upload(dict(mb, drop=drop))
    wk.G.zero_()
    wk.loss_buf.zero_()
    wk.forward_backward(d, wk.G, 0, 0)
    torch.cuda.synchronize()
    got_loss = float(wk.loss_buf[0].item())
    got_g = wk.G.cpu().numpy()
    # the dropped network differs from the plain one by far more than the tolerance, so agreeing with
    # the dropped oracle is a real statement about the masks and their scaling
    assert abs(float(want_loss) - float(plain_loss)) / abs(float(plain_loss)) > 5 * tol or rel(want_g, plain_g) > 5 * tol
    worst = ("loss", abs(got_loss - float(want_loss)) / abs(float(want_loss)))
    for name, off, r, c in O.param_layout(ocfg):
        e = rel(got_g[off:off + r * c], want_g[off:off + r * c])
        if e > worst[1]:
            worst = (name, e)
    print(f"{compute} L={L} B={len(lens)} p={drop['p']}: worst {worst[0]} {worst[1]:.2e}, |dropped - plain| grads {rel(want_g, plain_g):.2e}")
    assert worst[1] < tol, worst
    # a second pass with the same state gives the same bits; another stream number another result
    g1 = wk.G.clone()
    wk.forward_backward(d, wk.G, 0, 0)
    torch.cuda.synchronize()
    assert torch.equal(g1, wk.G)
    d2 = dict(d, drop=dict(drop, stream=drop["stream"] + 1))
    wk.forward_backward(d2, wk.G, 0, 0)
    torch.cuda.synchronize()
    assert not torch.equal(g1, wk.G)
    # and switching dropout off again restores the plain result
    d0 = dict(d, drop=None)
    wk.forward_backward(d0, wk.G, 0, 0)
    torch.cuda.synchronize()
    assert rel(wk.G.cpu().numpy(), plain_g) < tol
    wk.close()


def test_tiny_fp32_all_sites():
    run_case(synth.MODELS["tiny"], "fp32", [16, 32, 48, 64], 64, dict(p=0.1, seed=2024, stream=3), 11, 1e-4)


def test_tiny_fp32_heavy_dropout_and_ragged_lengths():
    run_case(synth.MODELS["tiny"], "fp32", [1, 7, 33, 60, 64], 64, dict(p=0.5, seed=7, stream=0xFFFFFFF0), 12, 1e-4)


def test_two_layer_bf16_short_sequences_fused_backward():
    model = dict(n_layers=2, hidden=256, n_heads=4, ffn=1024, vocab=2000, max_pos=128, ln_eps=1e-12)
    run_case(model, "bf16", [128, 100, 64, 17, 128, 96], 128, dict(p=0.1, seed=99, stream=1), 13, 2e-2)


def test_two_layer_bf16_long_sequences_two_kernel_backward():
    model = dict(n_layers=2, hidden=256, n_heads=4, ffn=1024, vocab=2000, max_pos=256, ln_eps=1e-12)
    run_case(model, "bf16", [256, 200, 129, 31], 256, dict(p=0.1, seed=5, stream=2), 14, 2e-2)


def test_bert_base_width_bf16():
    model = dict(synth.MODELS["bert_base"], n_layers=2)
    run_case(model, "bf16", [128] * 4 + [90, 128, 64, 128], 128, dict(p=0.1, seed=1234, stream=9), 15, 2e-2, ids="zipf")


def test_large_batch_runs_as_two_halves_with_the_masks_of_the_whole_batch():
    """4096 positions: the forward pass runs as two half-batches on two streams, each numbering its dropout elements
    from its offset in the whole batch; the oracle knows nothing of halves."""
    lens = [int(x) for x in synth.draw_lengths(synth.rng_for(40), 64, 5, 64)]
    run_case(synth.MODELS["tiny"], "fp32", lens, 64, dict(p=0.1, seed=77, stream=4), 16, 1e-4)
