"""GPU parity for the L1-quantised path (Equation 1 with p = 1; Appendix F.1): the exact
mean |c| must equal the oracle's bit for bit, as must the level bytes, their sums and the
vote; theta and momenta within 1e-6 relative / 1e-7 absolute."""
import numpy as np
import pytest
import torch

import oracle as orc
import paper_2411_16462_amd as lc
from harness import SENTINEL, Case, assert_close, guarded, untouched, words_of

pytestmark = pytest.mark.gpu

HP = dict(beta1=0.9, beta2=0.99, lr=1e-4, wd=0.1)


def heavy_tailed(case, seed, spread):
    """Laplace-like gradients with a heavy-tailed per-element scale (Section 4.1: update
    vectors look Laplacian, with outliers far above the mean)."""
    gen = torch.Generator(device="cuda").manual_seed(seed)
    shape = case.g.shape
    u = torch.rand(shape, generator=gen, device="cuda") - 0.5
    lap = -torch.sign(u) * torch.log1p(-2 * u.abs().clamp(max=0.499999))        # finite: rand() may return 0
    scale = torch.exp2(torch.randn(shape, generator=gen, device="cuda") * spread)
    case.g.copy_((lap * scale * 1e-3).to(case.g.dtype))
    case.snapshot()


def run_l1(case, L, step, tie=lc.LC_TIE_ZERO, n_m=0):
    n, W = case.n, case.W
    dev = case.device
    mean = torch.full((W,), -1.0, dtype=torch.float64, device=dev)
    ws = torch.full((W * lc.LC_L1_WORKSPACE_WORDS,), -1, dtype=torch.int64, device=dev)
    lc.lc_l1_mean_abs(case.g, case.g.stride(0), case.gd, case.m, case.m.stride(0), W, n, HP["beta1"], mean, ws)
    q = guarded(W, n, dev)
    lc.lc_l1_quantize_pack(case.g, case.g.stride(0), case.gd, case.m, case.m.stride(0), W, n, HP["beta1"], 1, HP["beta2"],
                           L, mean, q, q.stride(0))
    nw = (n + 63) // 64
    ksum, pos, nz = guarded(1, n, dev), guarded(1, nw * 8, dev), guarded(1, nw * 8, dev)
    lc.lc_level_sum_sign(q, q.stride(0), W, n, L, ksum, pos, nz, step, tie)
    ksum2 = guarded(1, n, dev)
    lc.lc_level_sum_apply(q, q.stride(0), W, n, L, ksum2, step, tie, case.theta, HP["lr"], HP["wd"], None, 0, None, 0,
                          lc.LC_F32, n_m, HP["beta2"])
    torch.cuda.synchronize()
    return dict(mean=mean.cpu().numpy(), q=q, ksum=ksum, ksum2=ksum2, pos=pos, nz=nz)


def check_l1(case, out, ref, L):
    n = case.n
    nw = (n + 63) // 64
    assert np.array_equal(out["mean"], ref["mean_abs"]), "mean |c| must be exact: %r vs %r" % (out["mean"], ref["mean_abs"])
    assert np.array_equal(out["q"][:, :n].cpu().numpy(), ref["fields"]), "level bytes"
    assert untouched(out["q"], n)
    for k in ("ksum", "ksum2"):
        assert np.array_equal(out[k][0, :n].cpu().numpy().astype(np.int32), ref["K"]), "summed level bytes"
        assert untouched(out[k], n)
    assert np.array_equal(words_of(out["pos"], nw)[0], ref["pos"]) and np.array_equal(words_of(out["nz"], nw)[0], ref["nz"])
    assert_close(case.theta.cpu().numpy(), ref["theta"], "theta")
    assert_close(case.m.cpu().numpy(), ref["m"], "momentum")


@pytest.mark.parametrize("n", [1, 3, 255, 256, 257, 4099, 65536 + 19, 300001])
@pytest.mark.parametrize("W,L", [(1, 127), (4, 31), (8, 15)])
def test_l1_sizes(n, W, L):
    case = Case(n, W, seed=20000 + n + W, m_spread=1.0)
    heavy_tailed(case, n + W, spread=2.0)
    step = 1 + n % 2
    ref = orc.step_l1(case.theta0, case.m0, case.g0, L=L, step=step, **HP)
    check_l1(case, run_l1(case, L, step), ref, L)


@pytest.mark.parametrize("g_dtype", ["f32", "bf16"])
@pytest.mark.parametrize("spread", [0.0, 6.0, 25.0])
def test_l1_dynamic_range(g_dtype, spread):
    """Narrow to extreme dynamic range inside single tiles (spread 25: magnitudes span
    hundreds of binary orders, so the lane-by-lane path of the exact sum runs), plus
    zeros and denormals."""
    n, W, L = 70000, 3, 15
    case = Case(n, W, seed=21000, g_dtype=g_dtype, m_scale=0.0 if spread > 10 else 1e-3)
    heavy_tailed(case, int(spread) + 5, spread)
    case.g[:, 1000:3000] = 0
    case.g[0, 5000:5004] = torch.tensor([1e-40, -1e-44, 3e-39, 0.0], device="cuda").to(case.g.dtype)
    case.snapshot()
    ref = orc.step_l1(case.theta0, case.m0, case.g0, L=L, step=2, tie=orc.TIE_ALT,
                      g_dtype=orc.BF16 if g_dtype == "bf16" else orc.F32, **HP)
    check_l1(case, run_l1(case, L, 2, lc.LC_TIE_ALT), ref, L)
    assert (ref["levels"] != 0).any() and np.abs(ref["levels"]).max() == L


def test_l1_all_zero_and_empty():
    n, W, L = 5000, 2, 15
    case = Case(n, W, seed=22000, m_scale=0.0)
    case.g.zero_()
    case.snapshot()
    ref = orc.step_l1(case.theta0, case.m0, case.g0, L=L, step=1, **HP)
    out = run_l1(case, L, 1)
    assert out["mean"].tolist() == [0.0, 0.0] and (ref["fields"] == L).all()
    check_l1(case, out, ref, L)
    mean = torch.full((W,), -1.0, dtype=torch.float64, device="cuda")
    ws = torch.zeros(W * lc.LC_L1_WORKSPACE_WORDS, dtype=torch.int64, device="cuda")
    lc.lc_l1_mean_abs(case.g, case.g.stride(0), case.gd, case.m, case.m.stride(0), W, 0, 0.9, mean, ws)
    torch.cuda.synchronize()
    assert mean.tolist() == [0.0, 0.0]


def test_l1_quantize_with_given_scale_and_range_rule():
    """The second pass on its own, fed the oracle's mean; and 2 L W <= 255."""
    n, W, L = 33333, 8, 15
    case = Case(n, W, seed=23000)
    heavy_tailed(case, 7, 3.0)
    c = np.stack([orc.local_c(case.m0[w], case.g0[w], HP["beta1"]) for w in range(W)])
    means = np.array([orc.mean_abs(c[w]) for w in range(W)]) * np.array([1, 0.5, 2, 1, 1, 3, 1, 0.25])
    q = guarded(W, n, "cuda")
    lc.lc_l1_quantize_pack(case.g, case.g.stride(0), case.gd, case.m, case.m.stride(0), W, n, HP["beta1"], 0, HP["beta2"], L,
                           torch.tensor(means, dtype=torch.float64, device="cuda"), q, q.stride(0))
    torch.cuda.synchronize()
    want = np.stack([orc.l1_levels(c[w], means[w], L) for w in range(W)]).astype(np.int16) + L
    assert np.array_equal(q[:, :n].cpu().numpy(), want.astype(np.uint8))
    assert np.array_equal(case.m.cpu().numpy(), case.m0)                     # update_m = 0
    rc = lc.lc_level_sum_sign(q, q.stride(0), 9, n, 15, None, None, None, 1, lc.LC_TIE_ZERO, check=False)
    assert rc == lc.LC_ERR_RANGE                                             # 9 * 30 = 270 > 255
    assert lc.lc_level_sum_sign(q, q.stride(0), 8, n, 0, None, None, None, 1, lc.LC_TIE_ZERO, check=False) == lc.LC_ERR_RANGE
    assert lc.lc_l1_quantize_pack(case.g, case.g.stride(0), case.gd, case.m, case.m.stride(0), W, n, 0.9, 0, 0.99, 128,
                                  torch.zeros(W, dtype=torch.float64, device="cuda"), q, q.stride(0),
                                  check=False) == lc.LC_ERR_RANGE


def test_l1_mean_is_reproducible_and_order_free():
    """Same bits on every run, and for a permutation of the elements."""
    n, W = 1 << 20, 2
    case = Case(n, W, seed=24000, m_scale=0.0)
    heavy_tailed(case, 3, 8.0)
    ws = torch.zeros(W * lc.LC_L1_WORKSPACE_WORDS, dtype=torch.int64, device="cuda")
    outs = []
    for rep in range(3):
        mean = torch.zeros(W, dtype=torch.float64, device="cuda")
        if rep == 2:
            perm = torch.randperm(n, device="cuda")
            case.g.copy_(case.g[:, perm])
        lc.lc_l1_mean_abs(case.g, case.g.stride(0), case.gd, case.m, case.m.stride(0), W, n, 0.0, mean, ws)
        outs.append(mean.cpu().numpy())
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])
    assert outs[0][0] == orc.mean_abs(case.g0[0])                            # beta1 = 0, m = 0: c = g
