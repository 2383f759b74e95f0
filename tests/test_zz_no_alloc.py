"""The entry point for callers that cannot allocate: hs_op_layernorm_bwd_noalloc keeps its partial column
sums in an array built into the library.  Checked through the C ABI against hs_op_layernorm_bwd (same
kernels, so the same bits) and against the oracle, on two calls in a row, the second on a smaller input."""
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


def rel(a, b):
    nb = np.linalg.norm(b)
    return np.linalg.norm(a - b) / nb if nb > 1e-12 else np.linalg.norm(a - b)


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def run_case(hs, mode, R, H, seed):
    dt = torch.bfloat16 if mode == 1 else torch.float32
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((R, H)) * 2 + 0.5).astype(np.float32)
    gain = (1 + 0.1 * rng.standard_normal(H)).astype(np.float32)
    dy = rng.standard_normal((R, H)).astype(np.float32)
    old = rng.standard_normal(H).astype(np.float32)
    xd, gd, dyd = (torch.from_numpy(a).cuda().to(dt) for a in (x, gain, dy))
    bias = torch.zeros(H, dtype=dt, device="cuda")
    y = torch.zeros(R, H, dtype=dt, device="cuda")
    stats = torch.zeros(2 * R, dtype=torch.float32, device="cuda")
    hs.hs_op_layernorm_fwd(mode, xd, gd, bias, y, stats, R, H, 1e-12)
    # every output buffer of both variants exists before the call under test: that call allocates nothing
    outs = []
    for _ in range(2):
        outs.append((torch.zeros(R, H, dtype=dt, device="cuda"),) + tuple(torch.from_numpy(old.copy()).cuda() for _ in range(3)))
    part = torch.zeros(hs.hs_op_layernorm_bwd_scratch(R, H), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    dx0, gg0, gb0, gs0 = outs[0]
    hs.hs_op_layernorm_bwd(mode, dyd, xd, stats, gd, dx0, gg0, gb0, gs0, 1.0, R, H, part)
    dx1, gg1, gb1, gs1 = outs[1]
    before = torch.cuda.memory_allocated()
    hs.hs_op_layernorm_bwd_noalloc(mode, dyd, xd, stats, gd, dx1, gg1, gb1, gs1, 1.0, R, H)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    # same kernels, same reduction order: the same bits as the entry point with a caller buffer
    for a, b in ((dx0, dx1), (gg0, gg1), (gb0, gb1), (gs0, gs1)):
        assert torch.equal(a, b)
    # and the oracle's LayerNorm backward on the values the kernel read
    def rounded(a):
        return torch.from_numpy(a).to(dt).float().numpy().astype(np.float64)
    xr, gr, dyr = rounded(x), rounded(gain), rounded(dy)
    _, cache = O.layer_norm_fwd(xr, gr, np.zeros(H), 1e-12)
    wdx, wdg, wdb = O.layer_norm_bwd(dyr, cache, gr)
    tol = 1e-5 if mode == 0 else 4e-3
    assert rel(host(dx1), wdx) < tol
    assert rel(host(gg1), old + wdg) < (1e-4 if mode == 0 else 5e-3)
    assert rel(host(gb1), old + wdb) < 1e-5
    assert rel(host(gs1), old + wdx.sum(0)) < (1e-4 if mode == 0 else 2e-2)


@pytest.mark.parametrize("mode", [0, 1])
def test_two_calls_in_a_row_second_smaller(hs, mode):
    run_case(hs, mode, 8192, 768, 11)      # uses every block of the row kernel: the whole scratch range of this H
    run_case(hs, mode, 203, 256, 12)       # smaller, ragged: stale partials of the first call lie beyond what it reads
    run_case(hs, mode, 5, 1024, 13)        # the widest row the scratch is sized for


def test_limits_are_errors(hs):
    t = torch.zeros(8, dtype=torch.float32, device="cuda")
    for R, H in ((4, 2048), (4, 96), (-1, 64)):
        with pytest.raises(hs.HsError):
            hs.hs_op_layernorm_bwd_noalloc(0, t, t, t, t, t, None, None, None, 0.0, R, H)
