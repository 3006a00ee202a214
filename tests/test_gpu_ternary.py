"""GPU parity for the ternary wire format (Appendix B.1: exact zeros travel as a second
plane): per-worker pos / nz planes, the vote sign(K+ - K-) and the fused apply."""
import numpy as np
import pytest
import torch

import oracle as orc
import paper_2411_16462_amd as lc
from harness import Case, assert_close, guarded, untouched, words_of

pytestmark = pytest.mark.gpu

HP = dict(beta1=0.9, beta2=0.99, lr=1e-4, wd=0.1)


def run(case, n_m=0):
    n, W = case.n, case.W
    nw = (n + 63) // 64
    pos, nz = guarded(W, nw * 8, case.device), guarded(W, nw * 8, case.device)
    lc.lc_local_update_pack_ternary(case.g, case.g.stride(0), case.gd, case.m, case.m.stride(0), W, n, HP["beta1"], 1,
                                    HP["beta2"], pos, nz, pos.stride(0) // 8)
    vp, vz = guarded(1, nw * 8, case.device), guarded(1, nw * 8, case.device)
    lc.lc_vote_ternary(pos, nz, pos.stride(0) // 8, W, n, vp, vz)
    lc.lc_vote_apply_ternary(pos, nz, pos.stride(0) // 8, W, n, case.theta, HP["lr"], HP["wd"], None, 0, None, 0, lc.LC_F32,
                             0, HP["beta2"])
    torch.cuda.synchronize()
    return pos, nz, vp, vz


def check(case, out, ref):
    pos, nz, vp, vz = out
    nw = (case.n + 63) // 64
    assert np.array_equal(words_of(pos, nw), ref["pos_w"]) and np.array_equal(words_of(nz, nw), ref["nz_w"])
    assert untouched(pos, nw * 8) and untouched(nz, nw * 8) and untouched(vp, nw * 8) and untouched(vz, nw * 8)
    assert np.array_equal(words_of(vp, nw)[0], ref["pos"]) and np.array_equal(words_of(vz, nw)[0], ref["nz"])
    assert_close(case.theta.cpu().numpy(), ref["theta"], "theta")
    assert_close(case.m.cpu().numpy(), ref["m"], "momentum")


@pytest.mark.parametrize("n", [1, 63, 64, 65, 1023, 1025, 4099, 70000])
@pytest.mark.parametrize("W", [1, 2, 3, 4, 8, 15, 16, 64, 255])
def test_ternary_sizes(n, W):
    if n > 5000 and W > 16:
        pytest.skip("large n with many workers adds nothing")
    case = Case(n, W, seed=30000 + n + W, m_scale=0.0)
    # many exact zeros: single workers, and whole columns
    zero = torch.rand(case.g.shape, device="cuda") < 0.3
    case.g[zero] = 0
    case.g[:, : min(n, 17)] = 0
    case.snapshot()
    ref = orc.step_ternary(case.theta0, case.m0, case.g0, **HP)
    assert (ref["s"] == 0).mean() > 0.2
    check(case, run(case), ref)


@pytest.mark.parametrize("g_dtype", ["f32", "bf16"])
def test_ternary_keeps_structural_zeros(g_dtype):
    """A parameter whose gradient and momentum are always zero (an unused embedding row,
    Appendix B.1) is left alone by the ternary format on every iteration, where the 1-bit
    format moves it by +-lr."""
    n, W = 9000, 4
    case = Case(n, W, seed=31000, g_dtype=g_dtype)
    case.m[:, 2000:3000] = 0
    case.g[:, 2000:3000] = 0
    case.snapshot()
    ref = orc.step_ternary(case.theta0, case.m0, case.g0, g_dtype=orc.BF16 if g_dtype == "bf16" else orc.F32, **HP)
    check(case, run(case), ref)
    assert (ref["u"][2000:3000] == 0).all()
    th = case.theta.cpu().numpy()[2000:3000].astype(np.float64)
    assert np.allclose(th, case.theta0[2000:3000].astype(np.float64) * (1 - 1e-4 * 0.1), rtol=1e-6, atol=1e-7)


def test_ternary_apply_with_momentum_stream_and_ignored_pos_bits():
    n, W = 20000, 5
    case = Case(n, W, seed=32000, m_scale=0.0)
    case.g[:, 100:400] = 0
    case.snapshot()
    ref = orc.step_ternary(case.theta0, case.m0, case.g0, **HP)
    nw = (n + 63) // 64
    pos, nz = guarded(W, nw * 8, case.device), guarded(W, nw * 8, case.device)
    lc.lc_local_update_pack_ternary(case.g, case.g.stride(0), case.gd, case.m, case.m.stride(0), W, n, HP["beta1"], 0,
                                    HP["beta2"], pos, nz, pos.stride(0) // 8)
    torch.cuda.synchronize()
    assert np.array_equal(case.m.cpu().numpy(), case.m0)
    # a pos bit whose nz bit is clear does not count
    stray = pos.clone()
    stray[:, :8] |= ~nz[:, :8]
    lc.lc_vote_apply_ternary(stray, nz, pos.stride(0) // 8, W, n, case.theta, HP["lr"], HP["wd"], case.m, case.m.stride(0),
                             case.g, case.g.stride(0), case.gd, 2, HP["beta2"])
    torch.cuda.synchronize()
    assert_close(case.theta.cpu().numpy(), ref["theta"], "theta")
    got = case.m.cpu().numpy()
    assert_close(got[:2], ref["m"][:2], "momentum")
    assert np.array_equal(got[2:], case.m0[2:])
