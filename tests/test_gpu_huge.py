"""Indexing beyond 2^32 elements: one worker row of n = 2^32 + 197 parameters (52 GB of
state) through update+pack, vote+apply and the plane-based apply.  Windows at the start,
across the 2^32 boundary and at the ragged end are compared with the oracle; population
counts tie the packed words to the applied update over the whole range."""
import numpy as np
import pytest
import torch

import oracle as orc
import paper_2411_16462_amd as lc
from harness import assert_close

pytestmark = pytest.mark.gpu

N = (1 << 32) + 64 * 3 + 5
HP = dict(beta1=0.9, beta2=0.99, lr=1e-4, wd=0.1)
CHUNK = 1 << 28


def fill_normal(t, scale, gen):
    for lo in range(0, t.numel(), CHUNK):
        hi = min(t.numel(), lo + CHUNK)
        t[lo:hi] = torch.randn(hi - lo, generator=gen, device="cuda") * scale


def test_rows_longer_than_2_to_32_elements():
    free, _ = torch.cuda.mem_get_info()
    if free < 80 << 30:
        pytest.skip("needs 80 GB of free device memory")
    gen = torch.Generator(device="cuda").manual_seed(0x2411)
    n, W, step = N, 1, 1
    nw = (n + 63) // 64
    theta = torch.empty(n, dtype=torch.float32, device="cuda")
    m = torch.empty((1, n), dtype=torch.float32, device="cuda")
    g = torch.empty((1, n), dtype=torch.float32, device="cuda")
    fill_normal(theta, 0.02, gen)
    fill_normal(m[0], 1e-3, gen)
    fill_normal(g[0], 1e-3, gen)
    g[0, ::1001] = 0                                                       # zeros for the zero rule
    m[0, ::1001] = 0
    q = torch.zeros((1, nw + 8), dtype=torch.int64, device="cuda")
    spans = [(0, 4096), ((1 << 32) - 2048, (1 << 32) + 128), (n - 197 - 1024, n)]
    keep = [(theta[lo:hi].cpu().numpy(), m[0, lo:hi].cpu().numpy(), g[0, lo:hi].cpu().numpy()) for lo, hi in spans]
    theta_before_sum = float(theta[-4096:].double().sum())

    lc.lc_local_update_pack(g, n, lc.LC_F32, m, n, W, n, HP["beta1"], 1, HP["beta2"], 1, q, q.stride(0) * 8, step,
                            lc.LC_ZERO_ALT)
    pos = torch.zeros(nw + 8, dtype=torch.int64, device="cuda")
    nz = torch.zeros(nw + 8, dtype=torch.int64, device="cuda")
    lc.lc_vote_1bit(q, q.stride(0), W, n, pos, nz, step, lc.LC_TIE_ZERO)
    theta2 = theta.clone()
    lc.lc_vote_apply_1bit(q, q.stride(0), W, n, step, lc.LC_TIE_ZERO, theta, HP["lr"], HP["wd"], None, 0, None, 0,
                          lc.LC_F32, 0, HP["beta2"])
    lc.lc_apply_update(theta2, pos, nz, n, HP["lr"], HP["wd"], None, 0, None, 0, lc.LC_F32, 0, HP["beta2"])
    torch.cuda.synchronize()
    assert torch.equal(theta, theta2), "fused and plane-based apply"
    del theta2
    assert torch.equal(pos[:nw], q[0, :nw]) and int(q[0, nw:].abs().max()) == 0        # W = 1: the vote is the row itself
    assert int(nz[nw - 1]) == (1 << (n % 64)) - 1 and bool((nz[:nw - 1] == -1).all())

    for (lo, hi), (th0, m0, g0) in zip(spans, keep):
        ref = orc.step_1bit(th0, m0[None], g0[None], step=step, **HP)
        assert lo % 64 == 0
        got = q[0, lo // 64:(hi + 63) // 64].cpu().numpy().view(np.uint64)
        assert np.array_equal(got, ref["words"][0]), "packed words in [%d, %d)" % (lo, hi)
        assert_close(theta[lo:hi].cpu().numpy(), ref["theta"], "theta in [%d, %d)" % (lo, hi))
        assert_close(m[0, lo:hi].cpu().numpy(), ref["m"][0], "momentum in [%d, %d)" % (lo, hi))
    assert float(theta[-4096:].double().sum()) != theta_before_sum                    # the tail did move


def test_l1_path_beyond_2_to_32_elements():
    """The exact mean over 2^32 + 197 elements against its closed form (gradients cycle
    through 1, 2, 3 times 2^-12, momenta zero, beta1 = 0, so c = g and the sum is a count),
    then levels, level sum and apply on windows against the oracle."""
    from fractions import Fraction
    free, _ = torch.cuda.mem_get_info()
    if free < 80 << 30:
        pytest.skip("needs 80 GB of free device memory")
    n, W, L, step = N, 1, 127, 2
    m = torch.zeros((1, n), dtype=torch.float32, device="cuda")
    g = torch.empty((1, n), dtype=torch.float32, device="cuda")
    theta = torch.empty(n, dtype=torch.float32, device="cuda")
    gen = torch.Generator(device="cuda").manual_seed(0x1646)
    fill_normal(theta, 0.02, gen)
    for lo in range(0, n, CHUNK):
        hi = min(n, lo + CHUNK)
        g[0, lo:hi] = ((torch.arange(lo, hi, device="cuda") % 3) + 1).to(torch.float32) * 2.0 ** -12
    g[0, 1 << 32] = -0.75                                                  # one large element past the boundary
    mean = torch.zeros(1, dtype=torch.float64, device="cuda")
    ws = torch.zeros(lc.LC_L1_WORKSPACE_WORDS, dtype=torch.int64, device="cuda")
    lc.lc_l1_mean_abs(g, n, lc.LC_F32, m, n, W, n, 0.0, mean, ws)
    counts = [len(range(r, n, 3)) for r in range(3)]
    total = sum(Fraction(c * (r + 1), 1 << 12) for r, c in enumerate(counts))
    total += Fraction(3, 4) - Fraction(((1 << 32) % 3) + 1, 1 << 12)
    want = float(total) / n                                                # one rounding of the sum, then the division
    assert mean.item() == want

    q = torch.zeros((1, n + 64), dtype=torch.uint8, device="cuda")
    ksum = torch.zeros(n + 64, dtype=torch.uint8, device="cuda")
    spans = [(0, 4096), ((1 << 32) - 2048, (1 << 32) + 128), (n - 197 - 1024, n)]
    th0 = [theta[lo:hi].cpu().numpy() for lo, hi in spans]
    lc.lc_l1_quantize_pack(g, n, lc.LC_F32, m, n, W, n, 0.0, 1, HP["beta2"], L, mean, q, q.stride(0))
    lc.lc_level_sum_apply(q, q.stride(0), W, n, L, ksum, step, lc.LC_TIE_ZERO, theta, HP["lr"], HP["wd"], None, 0, None, 0,
                          lc.LC_F32, 0, HP["beta2"])
    torch.cuda.synchronize()
    assert int(q[0, n:].max()) == 0 and int(ksum[n:].max()) == 0
    for (lo, hi), t0 in zip(spans, th0):
        gw = g[0, lo:hi].cpu().numpy()
        lev = orc.l1_levels(orc.local_c(np.zeros_like(gw), gw, 0.0), want, L)
        fields = (lev.astype(np.int16) + L).astype(np.uint8)
        assert np.array_equal(q[0, lo:hi].cpu().numpy(), fields), "levels in [%d, %d)" % (lo, hi)
        K, S, u = orc.level_sum_sign(fields[None], L, step, orc.TIE_ZERO)
        assert np.array_equal(ksum[lo:hi].cpu().numpy().astype(np.int32), K)
        assert_close(theta[lo:hi].cpu().numpy(), orc.apply(t0, u, HP["lr"], HP["wd"]), "theta in [%d, %d)" % (lo, hi))
        assert_close(m[0, lo:hi].cpu().numpy(), orc.momentum(np.zeros_like(gw), gw, HP["beta2"]), "momentum")
    assert int(q[0, 1 << 32]) == 0                                         # the large negative element clamps to -L
