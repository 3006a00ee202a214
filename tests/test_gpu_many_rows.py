"""The kernels that serve many 1-bit rows -- the pipelined vote kernel (W a multiple of 16)
and the 8-words-per-wave general kernel (W >= 32) -- over worker counts, ragged sizes, both
tie rules, single planes, momentum rows fused into the apply, and byte counts."""
import numpy as np
import pytest
import torch

import oracle as orc
import paper_2411_16462_amd as lc
from harness import Case, assert_close, clone_rows, guarded, hip_update_pack, oracle_step, untouched, words_of

pytestmark = pytest.mark.gpu

HP = dict(beta1=0.9, beta2=0.99, lr=1e-4, wd=0.1)


@pytest.mark.parametrize("W", [16, 32, 33, 48, 64, 80, 240])
@pytest.mark.parametrize("n", [1, 63, 64 * 5 + 1, 16384 + 77, 70001])
def test_vote_planes_fused_apply_and_counts(W, n):
    step = 1 + (n + W) % 2
    tie, otie = ((lc.LC_TIE_ZERO, orc.TIE_ZERO), (lc.LC_TIE_ALT, orc.TIE_ALT))[(n // 7 + W // 16) % 2]
    n_m = (W // 16 + n) % 3
    case = Case(n, W, seed=43000 + W + n, m_scale=0.0)               # m = 0: near-independent signs, many ties
    case.g[:, ::11] = 0                                              # whole columns of exact zeros
    case.snapshot()
    ref = oracle_step(case, HP, step, tie=otie, p=8)
    q, _ = hip_update_pack(case, HP, step, 1, update_m=False)
    nw = (n + 63) // 64
    assert np.array_equal(words_of(q, nw), np.stack([orc.pack_1bit(ref["b"][w]) for w in range(W)]))
    # planes: both, pos alone, nz alone
    pos, nz = guarded(1, nw * 8, case.device), guarded(1, nw * 8, case.device)
    pos1, nz1 = guarded(1, nw * 8, case.device), guarded(1, nw * 8, case.device)
    lc.lc_vote_1bit(q, q.stride(0) // 8, W, n, pos, nz, step, tie)
    lc.lc_vote_1bit(q, q.stride(0) // 8, W, n, pos1, None, step, tie)
    lc.lc_vote_1bit(q, q.stride(0) // 8, W, n, None, nz1, step, tie)
    # fused vote + apply with n_m momentum rows, and the same through the byte counts
    theta_b, m_b = case.theta.clone(), clone_rows(case.m)
    mg = lambda mm: (mm, mm.stride(0), case.g, case.g.stride(0)) if n_m else (None, 0, None, 0)
    lc.lc_vote_apply_1bit(q, q.stride(0) // 8, W, n, step, tie, case.theta, HP["lr"], HP["wd"], *mg(case.m), case.gd, n_m,
                          HP["beta2"])
    ksum = guarded(1, n, case.device)
    lc.lc_pbit_sum_apply(q, q.stride(0), 1, W, n, 8, ksum, step, tie, theta_b, HP["lr"], HP["wd"], *mg(m_b), case.gd, n_m,
                         HP["beta2"])
    torch.cuda.synchronize()
    for p_, z_ in ((pos, nz), (pos1, nz1)):
        assert np.array_equal(words_of(p_, nw)[0], ref["pos"]) and np.array_equal(words_of(z_, nw)[0], ref["nz"])
        assert untouched(p_, nw * 8) and untouched(z_, nw * 8)
    assert np.array_equal(ksum[0, :n].cpu().numpy().astype(np.int32), ref["K"]) and untouched(ksum, n)
    assert torch.equal(theta_b, case.theta) and torch.equal(m_b, case.m)          # both routes: the same bits
    assert_close(case.theta.cpu().numpy(), ref["theta"], "theta")
    got = case.m.cpu().numpy()
    assert_close(got[:n_m], ref["m"][:n_m], "momentum")
    assert np.array_equal(got[n_m:], case.m0[n_m:])
    if W % 2 == 0 and n > 1000:
        assert (ref["S"] == 0).any()
