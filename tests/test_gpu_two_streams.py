"""The library keeps no state of its own (lc_l1_mean_abs_static aside, which says so): the same
calls issued on two streams at once, on separate buffers, give what they give one after the
other -- each step against the oracle."""
import numpy as np
import pytest
import torch

import oracle as orc
import paper_2411_16462_amd as lc
from harness import Case, assert_close, guarded, words_of

pytestmark = pytest.mark.gpu
HP = dict(beta1=0.9, beta2=0.99, lr=1e-4, wd=0.1)


def test_two_streams_at_once():
    n, W, L = 700001, 8, 15
    nw = (n + 63) // 64
    cases = [Case(n, W, seed=31000 + k, m_spread=0.5) for k in range(2)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    bufs = []
    for c in cases:
        bufs.append(dict(q=guarded(W, nw * 8, "cuda"), lv=guarded(W, n, "cuda"), mean=torch.zeros(W, dtype=torch.float64, device="cuda"),
                         ws=torch.zeros(W * lc.LC_L1_WORKSPACE_WORDS, dtype=torch.int64, device="cuda"),
                         div=torch.zeros(1, dtype=torch.float64, device="cuda"), theta1=c.theta.clone(), m_pack=None))
    torch.cuda.synchronize()
    for rep in range(3):                       # interleave the launches of the two streams call by call
        for k in (0, 1):
            c, b, s = cases[k], bufs[k], streams[k]
            if rep == 0:
                lc.lc_momentum_divergence(c.m, c.m.stride(0), W, n, b["div"], stream=s)
                lc.lc_l1_mean_abs(c.g, c.g.stride(0), c.gd, c.m, c.m.stride(0), W, n, HP["beta1"], b["mean"], b["ws"], stream=s)
            elif rep == 1:
                lc.lc_l1_quantize_pack(c.g, c.g.stride(0), c.gd, c.m, c.m.stride(0), W, n, HP["beta1"], 0, HP["beta2"], L, b["mean"],
                                       b["lv"], b["lv"].stride(0), stream=s)
                lc.lc_local_update_pack(c.g, c.g.stride(0), c.gd, c.m, c.m.stride(0), W, n, HP["beta1"], 1, HP["beta2"], 1, b["q"],
                                        b["q"].stride(0), 3, lc.LC_ZERO_ALT, stream=s)
            else:
                lc.lc_vote_apply_1bit(b["q"], b["q"].stride(0) // 8, W, n, 3, lc.LC_TIE_ZERO, c.theta, HP["lr"], HP["wd"], None, 0,
                                      None, 0, lc.LC_F32, 0, HP["beta2"], stream=s)
                lc.lc_level_sum_apply(b["lv"], b["lv"].stride(0), W, n, L, None, 3, lc.LC_TIE_ZERO, b["theta1"], HP["lr"], HP["wd"],
                                      None, 0, None, 0, lc.LC_F32, 0, HP["beta2"], stream=s)
                lc.lc_momentum_avg(c.m, c.m.stride(0), W, n, stream=s)
    torch.cuda.synchronize()
    for c, b in zip(cases, bufs):
        ref = orc.step_1bit(c.theta0, c.m0, c.g0, step=3, **HP)
        assert np.array_equal(words_of(b["q"], nw), ref["words"])
        assert_close(c.theta.cpu().numpy(), ref["theta"], "theta (1-bit)")
        mean_m = orc.momentum_avg(ref["m"].astype(np.float32))
        assert_close(c.m.cpu().numpy(), np.broadcast_to(mean_m, (W, n)), "averaged momentum")
        l1 = orc.step_l1(c.theta0, c.m0, c.g0, L=L, step=3, **HP)
        assert np.array_equal(b["mean"].cpu().numpy(), l1["mean_abs"])
        assert np.array_equal(b["lv"][:, :n].cpu().numpy(), l1["fields"])
        assert_close(b["theta1"].cpu().numpy(), l1["theta"], "theta (levels)")
        d = orc.momentum_divergence(c.m0)
        assert abs(b["div"].item() - d) <= 1e-12 * d
