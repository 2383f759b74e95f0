"""Times every tiling of the library's bf16 GEMM kernel on the products of one BERT-base layer (64 x 128 tokens).

    python -m paper_2009_14783_amd.gemm_variants [--iters 50] [--step] [--variants -1,5,9] [--products "fwd ffn1,dx qkv"] [--cube]

Stand-alone: each product runs `iters` times back to back on fixed buffers with the epilogue it has in the training
step (bias, bias + residual, bias + GELU with both outputs, GELU' of a saved pre-activation, fp32 accumulate); the
table gives TFLOP/s per variant.  A variant that is not built with a product's epilogue, or cannot take its
contraction length, is served by the library's fallback kernel; the automatic choice is the row `auto`.
--step adds the whole training step (ms per step, 10 warm-up + 30 timed) with the variant forced for every product of the
forward pass and of the activation-gradient chain (the grouped weight-gradient launch keeps its own tiling).
--cube times 8192 x 8192 x 8192 products in the three operand layouts instead (no epilogue; fp32 output for the m-major layout).
--products keeps the named products only (for counter runs under a profiler).
Prints Markdown.  Needs the GPU and the built library; no oracle, no CPU path.
"""
from __future__ import annotations

import argparse
import time

import torch

from . import binding as hs
from . import synth
from .step import Worker

T, H, F = 8192, 768, 3072
# name, a_kmajor, b_kmajor, M, N, K, epilogue (0 none, 1 bias + residual, 2 bias + GELU, 3 GELU'), fp32 output
PRODUCTS = [
    ("fwd qkv", 1, 1, T, 3 * H, H, 0, 0), ("fwd out", 1, 1, T, H, H, 1, 0), ("fwd ffn1", 1, 1, T, F, H, 2, 0), ("fwd ffn2", 1, 1, T, H, F, 1, 0),
    ("dx ffn2", 1, 0, T, F, H, 3, 0), ("dx ffn1", 1, 0, T, H, F, 0, 0), ("dx out", 1, 0, T, H, H, 0, 0), ("dx qkv", 1, 0, T, H, 3 * H, 0, 0),
    ("dW ffn1", 0, 0, F, H, T, 0, 1), ("dW ffn2", 0, 0, H, F, T, 0, 1), ("dW out", 0, 0, H, H, T, 0, 1), ("dW qkv", 0, 0, 3 * H, H, T, 0, 1),
]
# A and B k-major; A k-major, B n-major; A and B m-major
CUBES = [("cube kk", 1, 1, 8192, 8192, 8192, 0, 0), ("cube kn", 1, 0, 8192, 8192, 8192, 0, 0), ("cube nn", 0, 0, 8192, 8192, 8192, 0, 1)]
NAMES = {-1: "auto", 0: "0: 128x128x32, 3/CU", 1: "1: 256x256x64", 2: "2: 256x192x64", 3: "3: 128x192x64, 2/CU", 4: "4: 256x128x32, 2/CU",
         5: "5: 128x128x64, 2/CU", 6: "6: 256x128x64", 7: "7: LDS-direct 128x128x32, 4 stages, 2/CU",
         8: "8: LDS-direct 128x128x32, 3 stages, 3/CU", 9: "9: LDS-direct 128x128x64, 2 stages, 2/CU",
         10: "10: LDS-direct 256x128x64, 3 stages", 11: "11: LDS-direct 256x128x64, 2 stages"}


def time_product(prod, iters, bufs):
    name, ak, bk, M, N, K, epi, cf = prod
    A, B, Cb, Cf, C2, aux, bias, ws = bufs
    lda = K if ak else M
    ldb = K if bk else N
    kw = dict(c_f32=cf, beta=1.0 if cf else 0.0)
    if not cf:
        kw.update(epi=epi, bias=None if epi == 3 else bias, aux=aux if epi in (1, 3) else None, ldaux=N if epi in (1, 3) else 0,
                  C2=C2 if epi == 2 else None)
    run = lambda: hs.hs_op_gemm(1, ak, bk, M, N, K, A, lda, B, ldb, Cf if cf else Cb, N, scratch=ws, scratch_bytes=ws.numel(), **kw)
    for _ in range(3):
        run()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        run()
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / iters
    return us, 2.0 * M * N * K / us / 1e6


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--iters", type=int, default=50)
    ap.add_argument("--step", action="store_true")
    ap.add_argument("--variants", default="", help="comma-separated variant numbers (-1: automatic); default: all")
    ap.add_argument("--products", default="", help="comma-separated product names; default: all")
    ap.add_argument("--cube", action="store_true")
    args = ap.parse_args()
    hs.lib()
    products = CUBES if args.cube else PRODUCTS
    if args.products:
        products = [p for p in products if p[0] in [q.strip() for q in args.products.split(",")]]
        if not products:
            raise SystemExit("--products: no such product")
    g = torch.Generator(device="cuda").manual_seed(1)
    n = max(p[3] * p[4] for p in products + [("", 0, 0, T, F, 0, 0, 0)])
    n = max(n, max(max(p[3], p[4]) * p[5] for p in products))
    A = (torch.randn(n, generator=g, device="cuda") * 0.5).to(torch.bfloat16)
    B = (torch.randn(n, generator=g, device="cuda") * 0.05).to(torch.bfloat16)
    aux = torch.randn(n, generator=g, device="cuda").to(torch.bfloat16)
    bufs = (A, B, torch.empty(n, dtype=torch.bfloat16, device="cuda"),
            torch.zeros(max([F * 3 * H] + [p[3] * p[4] for p in products if p[7]]), dtype=torch.float32, device="cuda"),
            torch.empty(n, dtype=torch.bfloat16, device="cuda"), aux, torch.zeros(max([F] + [p[4] for p in products]), dtype=torch.bfloat16, device="cuda"),
            torch.empty(96 << 20, dtype=torch.uint8, device="cuda"))
    variants = [int(v) for v in args.variants.split(",")] if args.variants else [-1] + list(range(12))
    for prod in products:      # untimed pass: clocks up, code loaded
        time_product(prod, 3, bufs)
    print("| variant | " + " | ".join(p[0] for p in products) + " | sum (us) |")
    print("|---|" + "---|" * (len(products) + 1))
    for v in variants:
        hs.hs_tune_gemm_variant(v)
        cells, tot = [], 0.0
        for prod in products:
            us, tf = time_product(prod, args.iters, bufs)
            cells.append(f"{tf:.0f}")
            tot += us
        print(f"| {NAMES[v]} | " + " | ".join(cells) + f" | {tot:.0f} |", flush=True)
    hs.hs_tune_gemm_variant(-1)
    if not args.step:
        return
    wl = synth.WORKLOADS[1]
    model = synth.MODELS[wl["model"]]
    cfg = hs.make_cfg(**model)
    theta = synth.init_params(hs.hs_param_layout(cfg), wl["seed"])
    worker = Worker(model, wl["compute"], theta)
    dev = [worker.upload(b) for b in synth.workload_micro_batches(1)]
    print("\n| variant | ms per step |\n|---|---|")
    for v in variants:
        hs.hs_tune_gemm_variant(v)
        for _ in range(10):
            worker.train_step(dev, wl["adam"])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(30):
            worker.train_step(dev, wl["adam"])
        torch.cuda.synchronize()
        print(f"| {NAMES[v]} | {(time.perf_counter() - t0) / 30 * 1e3:.3f} |", flush=True)
    hs.hs_tune_gemm_variant(-1)


if __name__ == "__main__":
    main()
