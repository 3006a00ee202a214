"""lc_l1_mean_abs_static, the entry point for callers that cannot allocate: its means must
equal lc_l1_mean_abs's bit for bit (the sum of |c| is exact, so the bar is equality) on two
calls in a row that share the library's static workspace, the second with a smaller input;
the means are also checked against the oracle.  Collected last among the test files."""
import numpy as np
import pytest
import torch

import oracle as orc
import paper_2411_16462_amd as lc
from harness import Case

pytestmark = pytest.mark.gpu

BETA1 = 0.9


def both(case, W, n):
    dev = case.device
    ws = torch.full((W * lc.LC_L1_WORKSPACE_WORDS,), -1, dtype=torch.int64, device=dev)
    ref = torch.full((W,), -1.0, dtype=torch.float64, device=dev)
    got = torch.full((W,), -2.0, dtype=torch.float64, device=dev)
    lc.lc_l1_mean_abs(case.g, case.g.stride(0), case.gd, case.m, case.m.stride(0), W, n, BETA1, ref, ws)
    lc.lc_l1_mean_abs_static(case.g, case.g.stride(0), case.gd, case.m, case.m.stride(0), W, n, BETA1, got)
    torch.cuda.synchronize()
    return got.cpu().numpy(), ref.cpu().numpy()


def test_static_workspace_matches_caller_workspace_twice():
    big = Case(300001, 8, seed=31000, m_spread=1.0)
    small = Case(4099, 3, seed=31001, g_dtype="bf16", m_spread=1.0)
    for case in (big, small):            # the second call finds the first call's sums in the array
        got, ref = both(case, case.W, case.n)
        assert np.array_equal(got, ref), "static workspace: %r vs %r" % (got, ref)
        want = np.array([orc.mean_abs(orc.local_c(case.m0[w], case.g0[w], BETA1, case.oracle_gd()))
                         for w in range(case.W)])
        assert np.array_equal(got, want), "oracle: %r vs %r" % (got, want)
    # an even smaller one: a sub-range and fewer workers of the first case
    got, ref = both(big, 2, 777)
    assert np.array_equal(got, ref)
    # and an empty range gives zeros
    got, ref = both(big, 5, 0)
    assert np.array_equal(got, ref) and not got.any()


def test_static_workspace_limits():
    case = Case(1000, 2, seed=31002)
    out = torch.zeros(lc.LC_L1_STATIC_MAX_W + 1, dtype=torch.float64, device="cuda")
    args = (case.g, case.g.stride(0), case.gd, case.m, case.m.stride(0))
    assert lc.lc_l1_mean_abs_static(*args, lc.LC_L1_STATIC_MAX_W + 1, 10, BETA1, out, check=False) == lc.LC_ERR_SIZE
    assert lc.lc_l1_mean_abs_static(*args, 0, 10, BETA1, out, check=False) == lc.LC_ERR_SIZE
    assert lc.lc_l1_mean_abs_static(*args, 2, 10, BETA1, None, check=False) == lc.LC_ERR_NULL
    torch.cuda.synchronize()
    assert not out.any().item()          # a refused call wrote nothing
