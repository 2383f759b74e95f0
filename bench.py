#!/usr/bin/env python3
"""Benchmark of the HetSeq training-step hot path on one MI355X.

A step is one pass of the whole path over one synthetic batch of the BERT-base workload
(64 sequences x 128 tokens under a max-tokens cap of 8192): batch formation on the host,
encoder forward, masked-LM loss, backward, accumulation into the flat fp32 gradient buffer,
normalisation by the global sample count, fused Adam.  Inputs are resident in HBM before the
timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W]      (defaults: 10 warm-up steps, 50 timed steps)

`ms_per_step` and `value` are the mean over the timed steps; `ms_per_step_median` and `ms_per_step_min` come from
events recorded around every step.  The headline workload cycles through four distinct seeded batches.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
CAL_COPY_BYTES = 256 << 20     # size of the calibration copy (bytes read = bytes written)


def algorithmic_flops(model, mbs):
    """Forward + backward (2x forward) flops of the micro-batches: per real token and layer
    24 H^2 + 4 L H (F = 4H, attention over the padded length of its batch), per masked token
    2 H^2 + 2 H V; recomputation inside attention backward is not counted."""
    H, V, NL = model["hidden"], model["vocab"], model["n_layers"]
    total = 0.0
    for mb in mbs:
        L = mb["ids"].shape[1]
        total += 3.0 * NL * mb["n_real_tokens"] * (24.0 * H * H + 4.0 * L * H)
        total += 3.0 * mb["mlm_pos"].size * (2.0 * H * H + 2.0 * H * V)
    return total


GEMM_SOURCES = ("gemm.hip", "gemm_dev.h", "gemm_wide.h", "gemm_dma.h", "gemm_wide_kk.hip", "gemm_wide_kn.hip", "gemm_wide_nn.hip")


def gemm_source_hash():
    """SHA-256 over the GEMM sources in the tree: counter summaries under profiles/ are only quoted while it matches."""
    import hashlib
    h = hashlib.sha256()
    for name in GEMM_SOURCES:
        h.update(open(os.path.join(ROOT, "paper_2009_14783_amd", "csrc", name), "rb").read())
    return h.hexdigest()


def recorded_counter(file_name, key, kernel_class):
    """A per-launch figure of a GEMM class from a committed counter summary under profiles/ (lines of the form
    `<key> <class> <value>` and `gemm_source_sha256: <hash>`), or None when the summary is missing or was taken with
    GEMM sources other than the ones in the tree."""
    try:
        text = open(os.path.join(ROOT, "profiles", file_name)).read()
        now = gemm_source_hash()
    except OSError:
        return None
    sha, value = None, None
    for line in text.splitlines():
        f = line.split()
        if len(f) == 2 and f[0] == "gemm_source_sha256:":
            sha = f[1]
        if len(f) == 3 and f[0] == key and f[1] == kernel_class:
            value = float(f[2])
    return value if sha == now else None


def recorded_traffic(kernel_class):
    """HBM-side bytes per launch (two profiler runs, FETCH_SIZE and WRITE_SIZE, scaled by the calibration copy)."""
    return recorded_counter("bench_bert_base_L128_hbm_traffic.md", "traffic_bytes_per_launch", kernel_class)


def recorded_mfma_busy(kernel_class):
    """Share of the CU-busy cycles in which the matrix pipes of the class's kernels were busy (SQ counters)."""
    return recorded_counter("bench_bert_base_L128_sq_counters.md", "mfma_busy", kernel_class)


def cpu_baseline(model, wl, theta, mbs, n_seq_sample=64):
    """The oracle, as it stands, on a bounded sample of the same workload: the first
    n_seq_sample sequences of the batch (all of them by default: about 12 s) through the identical
    step (forward, loss, backward, normalise, Adam over all parameters)."""
    from threadpoolctl import threadpool_info
    from oracle import hetseq_oracle as O
    ocfg = O.ModelCfg(**model)
    mb = mbs[0]
    L = mb["ids"].shape[1]
    keep = mb["mlm_pos"] < n_seq_sample * L
    sample = dict(ids=mb["ids"][:n_seq_sample], lens=mb["lens"][:n_seq_sample], mlm_pos=mb["mlm_pos"][keep],
                  mlm_label=mb["mlm_label"][keep])
    th = theta.copy()
    m, v = np.zeros_like(th), np.zeros_like(th)
    t0 = time.perf_counter()
    O.train_step(ocfg, th, m, v, 1, [sample], **wl["adam"])
    dt = time.perf_counter() - t0
    tokens = int(sample["lens"].sum())
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    return dict(value=tokens / dt, unit="tokens/s", cores=int(threads), kind="oracle",
                sample=f"{n_seq_sample} of the 64 sequences ({tokens} tokens), full 12-layer model, one whole step "
                       f"(fwd, loss, bwd, normalise, Adam) in fp32 NumPy: {dt:.1f} s",
                host_cores_available=len(os.sched_getaffinity(0)))


def pair_flops(model, mb):
    """Forward + backward (2x forward) algorithmic flops: per real source token and encoder layer 8 H^2 + 4 H F + 4 Ls H;
    per real target token and decoder layer 12 H^2 + 4 H F + 2 Lt H (causal: half the pairs) + 4 Ls H, plus the key/value
    projection of the encoder output 4 H^2 per source token and decoder layer; output projection 2 H V per target token."""
    H, F, V = model["hidden"], model["ffn"], model["vocab"]
    Ls, Lt = mb["src"].shape[1], mb["tgt_in"].shape[1]
    ns, nt = mb["n_src_tokens"], mb["n_tgt_tokens"]
    fwd = model["n_enc"] * ns * (8.0 * H * H + 4.0 * H * F + 4.0 * Ls * H)
    fwd += model["n_dec"] * (nt * (12.0 * H * H + 4.0 * H * F + 2.0 * Lt * H + 4.0 * Ls * H) + ns * 4.0 * H * H)
    fwd += nt * 2.0 * H * V
    return 3.0 * fwd


def main_pairs(args):
    """Second workload: one step of the Transformer-base translation model (section "Transformer Translation Model")."""
    import torch
    from paper_2009_14783_amd import binding as hs
    from paper_2009_14783_amd import synth
    from paper_2009_14783_amd.step import PairWorker
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    hs.lib()
    model = synth.S2S_MODELS["transformer_base"]
    adam = dict(lr=5e-4, beta1=0.9, beta2=0.98, eps=1e-9)
    cfg = hs.make_s2s_cfg(**model)
    theta = synth.init_params(hs.hs_s2s_param_layout(cfg), 1240)
    mb = synth.pair_workload()
    if args.dropout > 0.0:
        mb["drop"] = dict(p=args.dropout, seed=1240, stream=0)
    worker = PairWorker(model, "bf16", theta)
    d = worker.upload(mb)
    lengths = np.maximum(mb["src_lens"], mb["tgt_lens"]).astype(np.int32)

    def one_step():
        hs.hs_make_batches(lengths, 32, 4096, 1)      # batch formation under the cap (host); its batch is the uploaded one
        return worker.train_step([d], adam)

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        D = one_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms = 1e3 * dt / args.steps
    loss, nll = worker.reported_loss(D)
    hs.hs_profile_enable(worker.ctx, 1)
    prof = {}
    for _ in range(args.profile_steps):
        worker.forward_backward(d, worker.G, 0, 0)
        torch.cuda.synchronize()
        for k, e in hs.hs_profile_read(worker.ctx).items():
            q = prof.setdefault(k, dict(launches=0, ms=0.0, flops=0.0, bytes=0.0))
            for f in q:
                q[f] += e[f]
    hs.hs_profile_enable(worker.ctx, 0)
    kernels = {k: dict(launches_per_step=q["launches"] / args.profile_steps, ms_per_step=q["ms"] / args.profile_steps,
                       tflops=q["flops"] / (q["ms"] * 1e-3) / 1e12, gbs=q["bytes"] / (q["ms"] * 1e-3) / 1e9)
               for k, q in prof.items() if q["launches"] and q["ms"] > 0}
    gemm = [k for k in ("gemm_fwd", "gemm_dx", "gemm_dw") if k in kernels]
    dominant = max(gemm, key=lambda k: kernels[k]["ms_per_step"])
    dp = prof[dominant]
    achieved = dp["flops"] / (dp["ms"] * 1e-3) / 1e12
    flops = pair_flops(model, mb)
    tokens = mb["n_src_tokens"] + mb["n_tgt_tokens"]
    out = dict(metric="trained tokens/sec on 1 MI355X (Transformer-base translation step) + % peak bf16 MFMA",
               value=tokens * args.steps / dt, unit="tokens/s", n_gpus=1, steps=args.steps, warmup=args.warmup, ms_per_step=ms,
               higher_is_better=True, scaling="weak", vs_baseline=None, dtype="bf16", data="synthetic",
               config=dict(workload="Transformer-base translation step: 6 + 6 post-LN layers, hidden 512, 8 heads, FFN 2048, shared "
                                    "vocabulary 37000, label smoothing 0.1, Adam 0.9/0.98/1e-9; 128 sentence pairs in 32-position "
                                    "buffers per side (max-tokens 4096), Zipf(1.1) ids, bf16 compute with fp32 master weights",
                           tokens_per_step=tokens, source_tokens=mb["n_src_tokens"], target_tokens=mb["n_tgt_tokens"], params=worker.P,
                           dropout=args.dropout),
               whole_step_tflops=flops / (ms * 1e-3) / 1e12, whole_step_mfma_frac=flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
               loss=loss, nll=nll,
               roofline=dict(bound="mfma", kernel=dominant, achieved=achieved, peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                             frac=achieved / PEAK_BF16_TFLOPS, traffic=None,
                             algorithmic_bytes_per_launch=dp["bytes"] / dp["launches"], avg_launch_us=1e3 * dp["ms"] / dp["launches"],
                             launches_per_step=dp["launches"] / args.profile_steps,
                             measured=f"HIP events around every launch, on the launch stream, in {args.profile_steps} extra passes"),
               kernels=kernels)
    if not args.no_cpu_baseline:
        from threadpoolctl import threadpool_info
        from oracle import hetseq_oracle as O
        from oracle import seq2seq_oracle as S
        ocfg = S.S2SCfg(**model)
        n = 128
        sample = {k: (v[:n] if isinstance(v, np.ndarray) else v) for k, v in mb.items()}
        th, om, ov = theta.copy(), np.zeros_like(theta), np.zeros_like(theta)
        n_steps = 4
        t0 = time.perf_counter()
        for t in range(1, n_steps + 1):
            l, _, g, _, n_tok = S.micro_batch_grad(ocfg, th, sample, 0.1)
            O.normalize(g, n_tok)
            O.adam_step(th, om, ov, g, t, **adam)
        cdt = time.perf_counter() - t0
        stok = n_steps * int(sample["src_lens"].sum() + sample["tgt_lens"].sum())
        threads = max([q.get("num_threads", 1) for q in threadpool_info()] + [1])
        out["cpu_baseline"] = dict(value=stok / cdt, unit="tokens/s", cores=int(threads), kind="oracle",
                                   sample=f"all {n} sentence pairs of the batch, full model, {n_steps} whole steps ({stok} tokens) in "
                                          f"fp32 NumPy: {cdt:.1f} s", host_cores_available=len(os.sched_getaffinity(0)))
    worker.close()
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--profile-steps", type=int, default=3, help="extra steps with per-kernel event timing")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--dropout", type=float, default=0.0,
                    help="dropout rate at the model's four kinds of sites (the headline figure is taken without: 0)")
    ap.add_argument("--workload", choices=["bert_base", "bert_varlen", "bert_hetero", "bert_large", "transformer_base"], default="bert_base",
                    help="bert_base: the headline workload (64 x 128 tokens); bert_varlen: 4096 sequences of 64..512 tokens batched under a "
                         "16384-token cap, one step per batch; bert_hetero: micro-batches of 8, 24 and 56 sequences x 256 per step; "
                         "bert_large: BERT-large, four micro-batches of 32 x 512 per step; transformer_base: the translation model's step")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the path runs on ONE GPU; --gpus must be 1 (no collectives, no sharding)",
              file=sys.stderr)
        sys.exit(2)

    if args.workload == "transformer_base":
        return main_pairs(args)

    import torch
    from paper_2009_14783_amd import binding as hs
    from paper_2009_14783_amd import synth
    from paper_2009_14783_amd.step import Worker
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    hs.lib()                                             # fail loudly if the HIP library is missing

    widx = {"bert_base": 1, "bert_varlen": 2, "bert_hetero": 3, "bert_large": 4}[args.workload]
    wl = synth.WORKLOADS[widx]
    model = synth.MODELS[wl["model"]]
    cfg = hs.make_cfg(**model)
    theta = synth.init_params(hs.hs_param_layout(cfg), wl["seed"])
    # step_mbs[i]: the micro-batches of step i (steps cycle through the list)
    if widx == 2:      # one step per batch of the corpus, batches formed by the library's batcher
        corpus = synth.draw_lengths(synth.rng_for(wl["seed"]), 4096, 64, 512)
        seq, offs, pads = hs.hs_make_batches(corpus, 64, 16384, 0)
        step_mbs = [[synth.make_micro_batch(synth.rng_for(wl["seed"] + 100 + j), corpus[seq[offs[j]:offs[j + 1]]], int(pads[j]), model["vocab"],
                                            wl["ids"])] for j in range(len(pads))]
        lengths, cap = corpus, 16384
        if args.steps == 50:
            args.steps = len(step_mbs)        # the default run is one pass over the batch list
    else:
        step_mbs = [synth.workload_micro_batches(widx)]
        if widx == 1:      # the headline workload cycles through four distinct seeded batches of the same shape
            step_mbs += [synth.step_micro_batches(wl["seed"], t, [128] * 64, 128, model["vocab"], wl["ids"]) for t in (1, 2, 3)]
        lengths = np.concatenate([mb["lens"] for mb in step_mbs[0]]).astype(np.int32)
        cap = {1: 8192, 3: 256 * 88, 4: 16384 * 4}[widx]
    mbs = step_mbs[0]
    worker = Worker(model, wl["compute"], theta)
    if args.dropout > 0.0:
        for sm in step_mbs:
            for i, mb in enumerate(sm):
                mb["drop"] = dict(p=args.dropout, seed=wl["seed"], stream=i)
    step_dev = [[worker.upload(mb) for mb in sm] for sm in step_mbs]      # inputs resident in HBM before timing
    dev_batches = step_dev[0]
    n_list = len(step_dev)
    tokens_of = [int(sum(mb["n_real_tokens"] for mb in sm)) for sm in step_mbs]
    flops_of = [algorithmic_flops(model, sm) for sm in step_mbs]
    tokens_per_step = sum(tokens_of[i % n_list] for i in range(args.steps)) / args.steps
    flops_per_step = sum(flops_of[i % n_list] for i in range(args.steps)) / args.steps
    step_no = [0]

    def one_step():
        # a0: batch formation under the max-tokens cap (host, integer); the batches it yields are the
        # ones already uploaded
        hs.hs_make_batches(lengths, 64, cap, 0)
        worker.train_step(step_dev[step_no[0] % n_list], wl["adam"])
        step_no[0] += 1

    # One plain elementwise copy of known size (256 MiB read, 256 MiB written) before anything is timed:
    # under a counter-collecting profiler it gives the scale of the HBM byte counters.
    cal_src = torch.ones(CAL_COPY_BYTES // 4, dtype=torch.float32, device="cuda")
    cal_dst = torch.empty_like(cal_src)
    torch.mul(cal_src, 1.0, out=cal_dst)
    torch.cuda.synchronize()
    del cal_src, cal_dst

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    step_no[0] = 0
    # The timed region: exactly --steps steps between two synchronisations (the mean, `ms_per_step` and `value`); an
    # event on the stream the steps are launched on before the first and after every step gives the spread (every
    # other stream the library uses is joined to that stream before a call returns).
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        one_step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = 1e3 * dt / args.steps
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    ms_median = per_step[len(per_step) // 2] if len(per_step) % 2 else 0.5 * (per_step[len(per_step) // 2 - 1] + per_step[len(per_step) // 2])
    ms_min = per_step[0]
    last = step_dev[(args.steps - 1) % n_list]
    D = sum(d["n_seq"] for d in last)
    loss = worker.reported_loss(D)

    # per-kernel timing with HIP events on the launch stream, in extra steps of the same loop
    hs.hs_profile_enable(worker.ctx, 1)
    prof = {}
    adam_ms = []
    for ps in range(args.profile_steps):
        ev0, ev1, ev2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        n_total = worker.accumulate_micro_batches(step_dev[ps % n_list])
        ev0.record()
        hs.hs_grad_accum_normalize(worker.G, None, worker.P, 0, float(n_total))
        ev1.record()
        worker.t += 1
        hs.hs_adam_step(worker.w, worker.m, worker.v, worker.G, worker.w_lowp, worker.P, wl["adam"]["lr"],
                        wl["adam"]["beta1"], wl["adam"]["beta2"], wl["adam"]["eps"], 0.0, worker.t)
        ev2.record()
        torch.cuda.synchronize()
        adam_ms.append((ev0.elapsed_time(ev1), ev1.elapsed_time(ev2)))
        for k, e in hs.hs_profile_read(worker.ctx).items():
            p = prof.setdefault(k, dict(launches=0, ms=0.0, flops=0.0, bytes=0.0))
            for f in p:
                p[f] += e[f]
    hs.hs_profile_enable(worker.ctx, 0)
    P = worker.P
    prof["accum"] = dict(launches=len(adam_ms), ms=sum(a for a, _ in adam_ms), flops=1.0 * P * len(adam_ms),
                         bytes=8.0 * P * len(adam_ms))
    prof["adam"] = dict(launches=len(adam_ms), ms=sum(b for _, b in adam_ms), flops=12.0 * P * len(adam_ms),
                        bytes=30.0 * P * len(adam_ms))
    kernels = {}
    for k, p in prof.items():
        if p["launches"] == 0:
            continue
        sec = p["ms"] * 1e-3
        kernels[k] = dict(launches_per_step=p["launches"] / args.profile_steps, ms_per_step=p["ms"] / args.profile_steps,
                          tflops=p["flops"] / sec / 1e12 if sec > 0 else 0.0, gbs=p["bytes"] / sec / 1e9 if sec > 0 else 0.0)
    gemm_classes = [k for k in ("gemm_fwd", "gemm_dx", "gemm_dw") if k in kernels]
    roofline = None
    if gemm_classes:
        dominant = max(gemm_classes, key=lambda k: kernels[k]["ms_per_step"])
        dp = prof[dominant]
        achieved = dp["flops"] / (dp["ms"] * 1e-3) / 1e12
        gemm_flops = sum(prof[k]["flops"] for k in gemm_classes)
        gemm_ms = sum(prof[k]["ms"] for k in gemm_classes)
        roofline = dict(bound="mfma", kernel=dominant, achieved=achieved, peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                        frac=achieved / PEAK_BF16_TFLOPS, traffic=recorded_traffic(dominant) if widx == 1 else None,
                        mfma_busy=recorded_mfma_busy(dominant) if widx == 1 else None,
                        algorithmic_bytes_per_launch=dp["bytes"] / dp["launches"],
                        avg_launch_us=1e3 * dp["ms"] / dp["launches"],
                        launches_per_step=dp["launches"] / args.profile_steps,
                        all_gemms_tflops=gemm_flops / (gemm_ms * 1e-3) / 1e12,
                        all_gemms_frac=gemm_flops / (gemm_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                        measured="HIP events around every launch, on the launch stream, in "
                                 f"{args.profile_steps} extra steps after the timed region")

    shape_text = {
        1: "BERT-base-shaped step: 12 post-LN layers, hidden 768, 12 heads, FFN 3072, vocab 30522, tied MLM head; 64 sequences x 128 "
           "tokens (max-tokens cap 8192)",
        2: f"BERT-base-shaped model; 4096 sequences of 64..512 tokens in buckets of 64 under a cap of 16384 real tokens: {n_list} batches, "
           "one step per batch",
        3: "BERT-base-shaped model; per step three micro-batches of 8, 24 and 56 sequences x 256 tokens accumulated and normalised by 88",
        4: "BERT-large-shaped model (24 layers, hidden 1024, 16 heads, FFN 4096); per step four micro-batches of 32 sequences x 512 tokens "
           "accumulated and normalised by 128",
    }[widx]
    out = dict(metric="trained tokens/sec on 1 MI355X (BERT-base step) + % peak bf16 MFMA" if widx == 1 else
                      f"trained tokens/sec on 1 MI355X ({args.workload} step) + % peak bf16 MFMA",
               value=tokens_per_step * args.steps / dt, unit="tokens/s", n_gpus=1, steps=args.steps, warmup=args.warmup,
               ms_per_step=ms_per_step, ms_per_step_median=ms_median, ms_per_step_min=ms_min, distinct_batches=n_list,
               higher_is_better=True, scaling="weak", vs_baseline=None, dtype="bf16",
               data="synthetic",
               config=dict(workload=shape_text + ", Zipf(1.1) ids, 15% MLM targets, bf16 compute with fp32 master weights and accumulation",
                           tokens_per_step=int(tokens_per_step) if float(tokens_per_step).is_integer() else tokens_per_step,
                           mlm_targets=int(sum(d["M"] for d in last)),
                           global_batch=D, seq_len=int(last[0]["L"]), params=P, dropout=args.dropout),
               whole_step_tflops=flops_per_step / (ms_per_step * 1e-3) / 1e12,
               whole_step_mfma_frac=flops_per_step / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
               loss=loss, roofline=roofline, kernels=kernels)
    if not args.no_cpu_baseline and widx == 1:
        out["cpu_baseline"] = cpu_baseline(model, wl, theta, mbs)
    worker.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
