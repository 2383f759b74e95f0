"""Kernel-level parity on the GPU, each through the C ABI: GEMM (all layouts and epilogues, ragged
sizes), LayerNorm, attention, flat-buffer kernels, key mask.  References are NumPy float64 (the
oracle's own functions where it has them) on the same seeded inputs."""
import math

import numpy as np
import pytest

from oracle import hetseq_oracle as O

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hs():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2009_14783_amd import binding
    binding.lib()            # a missing library is a failure, not a skip
    return binding


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t if dtype is None else t.to(dtype)


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def rel(a, b):
    nb = np.linalg.norm(b)
    return np.linalg.norm(a - b) / nb if nb > 1e-12 else np.linalg.norm(a - b)


def act_dtype(mode):
    return torch.bfloat16 if mode == 1 else torch.float32


def rounded(a, mode):
    """The values the kernel actually reads: float32 or bfloat16-rounded."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(act_dtype(mode)).float().numpy().astype(np.float64)


GEMM_SHAPES = [(200, 136, 104), (128, 128, 32), (257, 72, 520), (24, 1000, 128), (64, 64, 8), (40, 72, 250)]
LAYOUTS = [(1, 1), (1, 0), (0, 0)]


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("ak,bk", LAYOUTS)
@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm_layouts_ragged_fp32_out(hs, mode, ak, bk, M, N, K):
    rng = np.random.default_rng(M * 7 + N * 3 + K + ak * 2 + bk)
    if mode == 1 and ak and bk and K % 8:
        pytest.skip("bf16 with both operands k-major needs K % 8 == 0 (checked in test_error_paths)")
    ld_pad = 8
    A = rng.standard_normal((M, K) if ak else (K, M)).astype(np.float32)
    B = rng.standard_normal((N, K) if bk else (K, N)).astype(np.float32)
    # padded leading dimensions, zero padding (the kernels may read the 8-element chunk that holds
    # the last valid element)
    Ap = np.zeros((A.shape[0], A.shape[1] + ld_pad + (-A.shape[1]) % 8), np.float32); Ap[:, :A.shape[1]] = A
    Bp = np.zeros((B.shape[0], B.shape[1] + ld_pad + (-B.shape[1]) % 8), np.float32); Bp[:, :B.shape[1]] = B
    dA, dB = dev(Ap, act_dtype(mode)), dev(Bp, act_dtype(mode))
    C0 = rng.standard_normal((M, N + 3)).astype(np.float32)
    dC = dev(C0)
    bias = rng.standard_normal(N).astype(np.float32)
    dbias = dev(bias, act_dtype(mode))
    Ar, Br = rounded(A, mode), rounded(B, mode)
    Am = Ar if ak else Ar.T
    Bm = Br if bk else Br.T
    want = Am @ Bm.T + rounded(bias, mode)[None, :]
    hs.hs_op_gemm(mode, ak, bk, M, N, K, dA, Ap.shape[1], dB, Bp.shape[1], dC, N + 3, c_f32=1, beta=0.0, bias=dbias)
    torch.cuda.synchronize()
    got = host(dC)
    assert rel(got[:, :N], want) < 2e-6
    assert np.array_equal(got[:, N:], C0[:, N:].astype(np.float64))          # nothing written outside N
    # accumulate: C = 0.5*C + A B^T
    hs.hs_op_gemm(mode, ak, bk, M, N, K, dA, Ap.shape[1], dB, Bp.shape[1], dC, N + 3, c_f32=1, beta=0.5)
    torch.cuda.synchronize()
    assert rel(host(dC)[:, :N], 0.5 * want + Am @ Bm.T) < 2e-6


@pytest.mark.parametrize("mode", [0, 1])
def test_gemm_epilogues(hs, mode):
    rng = np.random.default_rng(5)
    M, N, K = 192, 136, 64
    A = rng.standard_normal((M, K)).astype(np.float32) * 0.5
    B = rng.standard_normal((N, K)).astype(np.float32) * 0.5
    R = rng.standard_normal((M, N)).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    dt = act_dtype(mode)
    dA, dB, dR, dbias = dev(A, dt), dev(B, dt), dev(R, dt), dev(bias, dt)
    base = rounded(A, mode) @ rounded(B, mode).T + rounded(bias, mode)
    tol = 1e-5 if mode == 0 else 4e-3
    out = torch.zeros(M, N, dtype=dt, device="cuda")
    out2 = torch.zeros(M, N, dtype=dt, device="cuda")
    hs.hs_op_gemm(mode, 1, 1, M, N, K, dA, K, dB, K, out, N, bias=dbias, epi=1, aux=dR, ldaux=N)
    torch.cuda.synchronize()
    assert rel(host(out), base + rounded(R, mode)) < tol
    hs.hs_op_gemm(mode, 1, 1, M, N, K, dA, K, dB, K, out, N, bias=dbias, epi=2, C2=out2)
    torch.cuda.synchronize()
    assert rel(host(out), base) < tol
    assert rel(host(out2), O.gelu(base)) < tol
    hs.hs_op_gemm(mode, 1, 1, M, N, K, dA, K, dB, K, out, N, epi=3, aux=dR, ldaux=N)
    torch.cuda.synchronize()
    assert rel(host(out), (base - rounded(bias, mode)) * O.gelu_grad(rounded(R, mode))) < tol


def test_gemm_bf16_large_k_and_many_tiles(hs):
    """Several tiles in each direction with a ragged tail, at transformer-like sizes."""
    rng = np.random.default_rng(9)
    for ak, bk in LAYOUTS:
        M, N, K = 520, 392, 1000 if not (ak and bk) else 1024
        A = (rng.standard_normal((M, K) if ak else (K, M)) * 0.1).astype(np.float32)
        B = (rng.standard_normal((N, K) if bk else (K, N)) * 0.1).astype(np.float32)
        dA, dB = dev(A, torch.bfloat16), dev(B, torch.bfloat16)
        dC = torch.zeros(M, N, dtype=torch.float32, device="cuda")
        hs.hs_op_gemm(1, ak, bk, M, N, K, dA, A.shape[1], dB, B.shape[1], dC, N, c_f32=1)
        torch.cuda.synchronize()
        Ar, Br = rounded(A, 1), rounded(B, 1)
        want = (Ar if ak else Ar.T) @ (Br if bk else Br.T).T
        assert rel(host(dC), want) < 2e-6, (ak, bk)


@pytest.mark.parametrize("variant", [-1] + list(range(12)))
def test_gemm_every_tiling_ragged_edges_and_epilogues(hs, variant):
    """Every built tiling of the bf16 kernel (hs_tune_gemm_variant; -1: the automatic choice), each operand layout with the
    epilogues it serves, on a product with several tiles per direction, ragged last tiles in M and N, and a contraction that
    is (1024) or is not (1000) a whole number of k-tiles."""
    rng = np.random.default_rng(100 + variant)
    M, N = 520, 392
    tol = 4e-3
    hs.hs_tune_gemm_variant(variant)
    try:
        for K in (1024, 1000):
            for ak, bk in LAYOUTS:
                A = (rng.standard_normal((M, K) if ak else (K, M)) * 0.1).astype(np.float32)
                B = (rng.standard_normal((N, K) if bk else (K, N)) * 0.1).astype(np.float32)
                R = rng.standard_normal((M, N)).astype(np.float32)
                bias = rng.standard_normal(N).astype(np.float32)
                dA, dB, dR, dbias = (dev(a, torch.bfloat16) for a in (A, B, R, bias))
                Ar, Br = rounded(A, 1), rounded(B, 1)
                prod = (Ar if ak else Ar.T) @ (Br if bk else Br.T).T
                ws = torch.zeros(8 << 20, dtype=torch.uint8, device="cuda")
                if not ak:        # weight-gradient layout: fp32 output, accumulated
                    C0 = rng.standard_normal((M, N)).astype(np.float32)
                    dC = dev(C0)
                    hs.hs_op_gemm(1, ak, bk, M, N, K, dA, A.shape[1], dB, B.shape[1], dC, N, c_f32=1, beta=1.0, scratch=ws, scratch_bytes=ws.numel())
                    torch.cuda.synchronize()
                    assert rel(host(dC), C0.astype(np.float64) + prod) < 2e-6, (variant, K, ak, bk)
                    continue
                base = prod + rounded(bias, 1)
                out = torch.zeros(M, N, dtype=torch.bfloat16, device="cuda")
                out2 = torch.zeros(M, N, dtype=torch.bfloat16, device="cuda")
                hs.hs_op_gemm(1, ak, bk, M, N, K, dA, A.shape[1], dB, B.shape[1], out, N, bias=dbias)
                torch.cuda.synchronize()
                assert rel(host(out), base) < tol, (variant, K, ak, bk, "bias")
                hs.hs_op_gemm(1, ak, bk, M, N, K, dA, A.shape[1], dB, B.shape[1], out, N, bias=dbias, epi=1, aux=dR, ldaux=N)
                torch.cuda.synchronize()
                assert rel(host(out), base + rounded(R, 1)) < tol, (variant, K, ak, bk, "residual")
                if bk:
                    hs.hs_op_gemm(1, ak, bk, M, N, K, dA, A.shape[1], dB, B.shape[1], out, N, bias=dbias, epi=2, C2=out2)
                    torch.cuda.synchronize()
                    assert rel(host(out), base) < tol and rel(host(out2), O.gelu(base)) < tol, (variant, K, ak, bk, "gelu")
                else:
                    hs.hs_op_gemm(1, ak, bk, M, N, K, dA, A.shape[1], dB, B.shape[1], out, N, epi=3, aux=dR, ldaux=N)
                    torch.cuda.synchronize()
                    assert rel(host(out), prod * O.gelu_grad(rounded(R, 1))) < tol, (variant, K, ak, bk, "gelu'")
    finally:
        hs.hs_tune_gemm_variant(-1)


def test_gemm_variant_out_of_range_is_an_error(hs):
    for v in (-2, 12, 1000):
        with pytest.raises(hs.HsError):
            hs.hs_tune_gemm_variant(v)
    hs.hs_tune_gemm_variant(-1)


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("R,H", [(37, 128), (1030, 768), (5, 1024)])
def test_layernorm_fwd_bwd(hs, mode, R, H):
    rng = np.random.default_rng(R + H)
    dt = act_dtype(mode)
    x = (rng.standard_normal((R, H)) * 2 + 0.5).astype(np.float32)
    gain = (1 + 0.1 * rng.standard_normal(H)).astype(np.float32)
    bias = (0.1 * rng.standard_normal(H)).astype(np.float32)
    dy = rng.standard_normal((R, H)).astype(np.float32)
    dx_, dg_, db_ = dev(x, dt), dev(gain, dt), dev(bias, dt)
    y = torch.zeros(R, H, dtype=dt, device="cuda")
    stats = torch.zeros(2 * R, dtype=torch.float32, device="cuda")
    hs.hs_op_layernorm_fwd(mode, dx_, dg_, db_, y, stats, R, H, 1e-12)
    torch.cuda.synchronize()
    xr, gr, br, dyr = rounded(x, mode), rounded(gain, mode), rounded(bias, mode), rounded(dy, mode)
    want, cache = O.layer_norm_fwd(xr, gr, br, 1e-12)
    tol = 1e-5 if mode == 0 else 4e-3
    assert rel(host(y), want) < tol
    assert rel(host(stats)[:R], xr.mean(-1)) < 1e-5
    assert rel(host(stats)[R:], cache[1][:, 0]) < 1e-5
    ddy = dev(dy, dt)
    dxo = torch.zeros(R, H, dtype=dt, device="cuda")
    part = torch.zeros(hs.hs_op_layernorm_bwd_scratch(R, H), dtype=torch.uint8, device="cuda")
    old = rng.standard_normal(H).astype(np.float32)
    gg, gb, gs = dev(old.copy()), dev(old.copy()), dev(old.copy())
    hs.hs_op_layernorm_bwd(mode, ddy, dx_, stats, dg_, dxo, gg, gb, gs, 1.0, R, H, part)
    torch.cuda.synchronize()
    wdx, wdg, wdb = O.layer_norm_bwd(dyr, cache, gr)
    assert rel(host(dxo), wdx) < tol
    assert rel(host(gg), old + wdg) < (1e-4 if mode == 0 else 5e-3)
    assert rel(host(gb), old + wdb) < 1e-5
    assert rel(host(gs), old + wdx.sum(0)) < (1e-4 if mode == 0 else 2e-2)
    # beta = 0 overwrites
    hs.hs_op_layernorm_bwd(mode, ddy, dx_, stats, dg_, dxo, gg, gb, None, 0.0, R, H, part)
    torch.cuda.synchronize()
    assert rel(host(gb), wdb) < 1e-5


def attention_reference(qkv, lens, B, L, A):
    H = A * 64
    q, k, v = (qkv[:, j * H:(j + 1) * H].reshape(B, L, A, 64).transpose(0, 2, 1, 3) for j in range(3))
    s = q @ k.transpose(0, 1, 3, 2) / 8.0
    valid = O.key_mask(lens, L).astype(bool)
    s = np.where(valid[:, None, None, :], s, -np.inf)
    mx = s.max(-1, keepdims=True)
    e = np.exp(s - mx)
    z = e.sum(-1, keepdims=True)
    p = e / z
    ctx = (p @ v).transpose(0, 2, 1, 3).reshape(B * L, H)
    lse = (mx + np.log(z))[..., 0]
    return q, k, v, p, ctx, lse, valid


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("B,L,A,lens", [(3, 64, 2, [64, 1, 37]), (2, 136, 3, [136, 70]), (1, 8, 1, [5]),
                                        (3, 512, 2, [512, 300, 33]), (2, 256, 1, [129, 256]), (3, 128, 2, [128, 77, 31]), (2, 104, 1, [104, 97])])
def test_attention_fwd_bwd(hs, mode, B, L, A, lens):
    rng = np.random.default_rng(B * L + A)
    H = A * 64
    dt = act_dtype(mode)
    qkv = rng.standard_normal((B * L, 3 * H)).astype(np.float32)
    dctx = rng.standard_normal((B * L, H)).astype(np.float32)
    lens_np = np.asarray(lens, dtype=np.int32)
    valid_rows = O.key_mask(lens_np, L).astype(bool).reshape(-1)
    dctx[~valid_rows] = 0.0                      # padded rows carry no gradient in the real path
    dqkv_, dl = dev(qkv, dt), dev(lens_np)
    ctx = torch.zeros(B * L, H, dtype=dt, device="cuda")
    lse = torch.zeros(B * A * L, dtype=torch.float32, device="cuda")
    hs.hs_op_attention_fwd(mode, dqkv_, dl, B, L, A, ctx, lse)
    torch.cuda.synchronize()
    qkvr = rounded(qkv, mode)
    q, k, v, p, wctx, wlse, valid = attention_reference(qkvr, lens_np, B, L, A)
    tol = 2e-5 if mode == 0 else 5e-3
    assert rel(host(ctx)[valid_rows], wctx[valid_rows]) < tol
    vr = np.broadcast_to(valid[:, None, :], (B, A, L))
    assert rel(host(lse).reshape(B, A, L)[vr], wlse[vr]) < 1e-5
    assert np.all(np.isfinite(host(ctx)))
    # backward
    dO = rounded(dctx, mode).reshape(B, L, A, 64).transpose(0, 2, 1, 3)
    # the kernel reads its own rounded ctx for the row dot products; the reference uses the exact one
    dv = p.transpose(0, 1, 3, 2) @ dO
    dp = dO @ v.transpose(0, 1, 3, 2)
    ds = p * (dp - (dp * p).sum(-1, keepdims=True))
    dq = ds @ k / 8.0
    dk = ds.transpose(0, 1, 3, 2) @ q / 8.0
    want = np.concatenate([a.transpose(0, 2, 1, 3).reshape(B * L, H) for a in (dq, dk, dv)], axis=1)
    want[~valid_rows] = 0.0
    out = torch.full((B * L, 3 * H), 7.0, dtype=dt, device="cuda")
    dvec = torch.zeros(B * A * L, dtype=torch.float32, device="cuda")
    hs.hs_op_attention_bwd(mode, dqkv_, ctx, lse, dev(dctx, dt), dl, B, L, A, out, dvec)
    torch.cuda.synchronize()
    got = host(out)
    assert np.all(got[~valid_rows] == 0.0)
    assert rel(got, want) < (5e-5 if mode == 0 else 1e-2)


def test_key_mask_bit_exact(hs):
    rng = np.random.default_rng(3)
    B, L = 37, 136
    lens = rng.integers(1, L + 1, size=B).astype(np.int32)
    out = torch.zeros(B * L, dtype=torch.uint8, device="cuda")
    hs.hs_key_mask(dev(lens), B, L, out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy().reshape(B, L), O.key_mask(lens, L))


@pytest.mark.parametrize("n", [1, 7, 4096, 1_000_003])
def test_accumulate_normalize_and_dummy(hs, n):
    rng = np.random.default_rng(n)
    G0 = rng.standard_normal(n).astype(np.float32)
    g = rng.standard_normal(n).astype(np.float32)
    G = dev(G0.copy())
    hs.hs_grad_accum_normalize(G, dev(g), n, 0, 0.0)
    torch.cuda.synchronize()
    assert np.array_equal(G.cpu().numpy(), G0 + g)                       # one fp32 add: bit exact
    # dummy batch: g is poison and must not be read; G bit-identical
    before = G.cpu().numpy().copy()
    poison = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    hs.hs_grad_accum_normalize(G, poison, n, 1, 0.0)
    torch.cuda.synchronize()
    assert G.cpu().numpy().tobytes() == before.tobytes()
    hs.hs_grad_accum_normalize(G, None, n, 0, 88.0)
    torch.cuda.synchronize()
    want = O.normalize(before.copy(), 88)
    np.testing.assert_allclose(G.cpu().numpy(), want, rtol=2e-7, atol=0)
    with pytest.raises(hs.HsError):
        hs.hs_grad_accum_normalize(G, None, n, 0, -1.0)


@pytest.mark.parametrize("n", [5, 1_000_003])
def test_adam_matches_oracle_over_steps(hs, n):
    rng = np.random.default_rng(n + 1)
    w0 = (1e-3 * rng.standard_normal(n)).astype(np.float32)
    w, m, v = dev(w0.copy()), torch.zeros(n, device="cuda"), torch.zeros(n, device="cuda")
    wl = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    ow, om, ov = w0.astype(np.float64), np.zeros(n), np.zeros(n)
    for t in range(1, 4):
        g = (rng.standard_normal(n) * 10.0 ** rng.integers(-6, 1, size=n)).astype(np.float32)
        g[: min(n, 3)] = 0.0
        hs.hs_adam_step(w, m, v, dev(g), wl, n, 1e-4, 0.9, 0.999, 1e-8, 0.01 if t == 3 else 0.0, t)
        O.adam_step(ow, om, ov, g.astype(np.float64), t, 1e-4, 0.9, 0.999, 1e-8, 0.01 if t == 3 else 0.0)
        torch.cuda.synchronize()
        assert rel(host(m), om) < 1e-6 and rel(host(v), ov) < 1e-6
        assert rel(host(w) - w0, ow - w0) < 1e-4
        assert rel(host(w), ow) < 1e-6
        assert torch.equal(wl, w.to(torch.bfloat16))                      # nearest-even copy
    with pytest.raises(hs.HsError):
        hs.hs_adam_step(w, m, v, w, None, n, 1e-4, 0.9, 0.999, 1e-8, 0.0, 0)


def test_error_paths_launch_nothing(hs):
    a = torch.zeros(64, 64, dtype=torch.bfloat16, device="cuda")
    c = torch.zeros(64, 64, dtype=torch.float32, device="cuda")
    with pytest.raises(hs.HsError):                 # both k-major, K not a multiple of 8
        hs.hs_op_gemm(1, 1, 1, 8, 8, 12, a, 64, a, 64, c, 64, c_f32=1)
    with pytest.raises(hs.HsError):                 # misaligned leading dimension
        hs.hs_op_gemm(1, 1, 1, 8, 8, 8, a, 12, a, 64, c, 64, c_f32=1)
    with pytest.raises(hs.HsError):                 # epilogue without its operand
        hs.hs_op_gemm(1, 1, 1, 8, 8, 8, a, 64, a, 64, c, 64, c_f32=1, epi=1)
    with pytest.raises(hs.HsError):                 # hidden not supported
        hs.hs_op_layernorm_fwd(0, c, c, c, c, c, 4, 96, 1e-12)
    torch.cuda.synchronize()
    assert float(c.abs().sum()) == 0.0


@pytest.mark.parametrize("ak,bk,M,N,K,cf", [(0, 0, 768, 264, 4104, 1), (1, 0, 200, 136, 30522, 0), (1, 1, 130, 72, 2048, 1)])
def test_gemm_split_k_with_scratch(hs, ak, bk, M, N, K, cf):
    """Few output tiles and a long contraction: the contraction is split over workgroups and the fp32
    partial sums are added in a fixed order; the result must not depend on that (beyond fp32 rounding)
    and must be bit-identical from run to run."""
    rng = np.random.default_rng(K)
    A = (rng.standard_normal((M, K) if ak else (K, M)) * 0.1).astype(np.float32)
    B = (rng.standard_normal((N, K) if bk else (K, N)) * 0.1).astype(np.float32)
    pad = lambda X: np.pad(X, ((0, 0), (0, (-X.shape[1]) % 8 + 8)))
    Ap, Bp = pad(A), pad(B)
    dA, dB = dev(Ap, torch.bfloat16), dev(Bp, torch.bfloat16)
    bias = rng.standard_normal(N).astype(np.float32)
    scratch = torch.empty(32 << 20, dtype=torch.uint8, device="cuda")
    outs = []
    for _ in range(2):
        C0 = rng.standard_normal((M, N)).astype(np.float32) if cf else np.zeros((M, N), np.float32)
        dC = dev(C0, torch.float32 if cf else torch.bfloat16)
        hs.hs_op_gemm(1, ak, bk, M, N, K, dA, Ap.shape[1], dB, Bp.shape[1], dC, N, c_f32=cf, beta=1.0 if cf else 0.0,
                      bias=dev(bias, torch.bfloat16), scratch=scratch, scratch_bytes=scratch.numel())
        torch.cuda.synchronize()
        Ar, Br = rounded(A, 1), rounded(B, 1)
        want = (Ar if ak else Ar.T) @ (Br if bk else Br.T).T + rounded(bias, 1) + (C0 if cf else 0.0)
        assert rel(host(dC), want) < (3e-6 if cf else 4e-3)
        outs.append(host(dC) - (C0 if cf else 0.0))
    if not cf:
        assert np.array_equal(outs[0], outs[1])
