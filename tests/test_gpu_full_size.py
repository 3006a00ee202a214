"""Full-size parity: the five benchmark workloads, run exactly as bench.py runs them
(same buffers, same C-ABI calls, same launch configuration), checked against the CPU
oracle on sampled windows -- the first and the last elements and random 64-aligned
windows in between -- plus properties that hold over the whole range."""
import numpy as np
import pytest
import torch

import bench
import oracle as orc
import paper_2411_16462_amd as lc
from harness import assert_close, g_host
from paper_2411_16462_amd import synth

pytestmark = pytest.mark.gpu

WINDOW = 4096
N_RANDOM_WINDOWS = 24


def windows(n, seed):
    rng = np.random.default_rng(seed)
    spans = [(0, min(n, WINDOW)), (max(0, (n - WINDOW) // 64 * 64), n)]
    for lo in rng.integers(0, max(1, n // 64 - WINDOW // 64), N_RANDOM_WINDOWS):
        spans.append((int(lo) * 64, min(n, int(lo) * 64 + WINDOW)))
    return spans


def popcount64(x):
    """Per-element population count of an int64 tensor (plain torch integer ops)."""
    m1, m2, m4 = 0x5555555555555555, 0x3333333333333333, 0x0F0F0F0F0F0F0F0F
    x = x - ((x >> 1) & m1)
    x = (x & m2) + ((x >> 2) & m2)
    x = (x + (x >> 4)) & m4
    return ((x * 0x0101010101010101) >> 56) & 0xFF


def host_rows(t, lo, hi):
    return t[:, lo:hi].cpu().numpy()


@pytest.mark.parametrize("name", ["c0", "c1", "c2", "c3"])
def test_training_workloads(name):
    wl = synth.workload(name)
    kernels, st, step_no = bench.build_step(wl, torch, lc, synth)
    n, W = wl.n, wl.W
    theta0 = st["theta"].clone()
    m0 = torch.empty((W, n), dtype=torch.float32, device="cuda")
    m0.copy_(st["m"])
    for k in kernels:
        k.fn()
    torch.cuda.synchronize()
    gd = orc.BF16 if wl.g_dtype == "bf16" else orc.F32
    hp = dict(beta1=wl.beta1, beta2=wl.beta2, lr=wl.lr, wd=wl.wd, step=step_no[0], g_dtype=gd)
    C = lc.lc_container_bits(wl.p)
    ties = 0
    for lo, hi in windows(n, wl.seed):
        th, mm = theta0[lo:hi].cpu().numpy(), host_rows(m0, lo, hi)
        gg = g_host(st["g"][:, lo:hi])
        if wl.mode == "1bit":
            ref = orc.step_1bit(th, mm, gg, **hp)
            got = st["q"][:, lo // 64:(hi + 63) // 64].cpu().numpy().view(np.uint64)
            assert np.array_equal(got, ref["words"]), "%s: packed words in [%d, %d)" % (name, lo, hi)
        else:
            ref = orc.step_pbit(th, mm, gg, p=wl.p, **hp)
            b0, b1 = lo * C // 8, (hi * C + 7) // 8
            assert np.array_equal(st["q"][:, b0:b1].cpu().numpy(), ref["fields"]), "%s: fields" % name
            assert np.array_equal(st["sum_out"][b0:b1].cpu().numpy(), ref["sum_fields"]), "%s: field sums" % name
        ties += int((ref["u"] == 0).sum())
        assert_close(st["theta"][lo:hi].cpu().numpy(), ref["theta"], "%s: theta in [%d, %d)" % (name, lo, hi))
        m_ref = ref["m"]
        if wl.momentum_avg:
            m_ref = np.broadcast_to(orc.momentum_avg(m_ref.astype(np.float32)), m_ref.shape)
        assert_close(host_rows(st["m"], lo, hi), m_ref, "%s: momentum in [%d, %d)" % (name, lo, hi))
    # whole-range properties
    d = (st["theta"] - theta0 * (1.0 - wl.lr * wl.wd)) / wl.lr            # = -u up to rounding
    assert float((d - d.round()).abs().max()) < 1e-2 and float(d.abs().max()) < 1.01
    u_all = -d.round()
    if wl.mode == "1bit":
        # unanimous workers decide the vote: all bits set -> u = +1, none set -> u = -1
        nw = (n + 63) // 64
        q = st["q"][:, :nw]
        all_set, any_set = q[0].clone(), q[0].clone()
        for w in range(1, W):
            all_set &= q[w]
            any_set |= q[w]
        shifts = torch.arange(64, device="cuda", dtype=torch.int64)
        for lo in range(0, nw, 1 << 22):                                   # chunks of 4M words
            hi = min(nw, lo + (1 << 22))
            a = ((all_set[lo:hi, None] >> shifts) & 1).view(-1)[: min(n, hi * 64) - lo * 64].bool()
            o = ((any_set[lo:hi, None] >> shifts) & 1).view(-1)[: min(n, hi * 64) - lo * 64].bool()
            uu = u_all[lo * 64: min(n, hi * 64)]
            assert bool((uu[a] == 1).all()) and bool((uu[~o] == -1).all())
    else:
        # the stored counts K and the applied update agree everywhere: u = sign(2K - W)
        assert C == 4
        fb = (n + 1) // 2
        by = st["sum_out"][:fb].to(torch.int16)
        K = torch.stack([by & 0xF, by >> 4], 1).view(-1)[:n]
        assert int(K.max()) <= W
        assert bool((torch.sign(2 * K - W).to(torch.float32) == u_all).all())
    if wl.momentum_avg:
        assert bool((st["m"] == st["m"][0]).all())
    assert ties >= 0


def test_reduction_only_workload():
    """N = 1.3e9, 64 pre-packed rows: majority vote + apply (one momentum stream), then
    the p = 7 sum of signs with the counts written as bytes."""
    wl = synth.workload("c4")
    kernels, st, step_no = bench.build_step(wl, torch, lc, synth)
    n, W = wl.n, wl.W
    nw = (n + 63) // 64
    q = st["q"]
    theta0, m0 = st["theta"].clone(), st["m"].clone()
    for k in kernels:
        k.fn()
    torch.cuda.synchronize()
    theta1, m1 = st["theta"].clone(), st["m"].clone()
    # second variant on fresh copies of the state: p = 7 sum + apply with counts out
    st["theta"].copy_(theta0)
    st["m"].copy_(m0)
    ksum = torch.zeros(n, dtype=torch.uint8, device="cuda")
    lc.lc_pbit_sum_apply(q, q.stride(0) * 8, 1, W, n, wl.p, ksum, step_no[0], lc.LC_TIE_ZERO, st["theta"], wl.lr, wl.wd,
                         st["m"], st["m"].stride(0), st["g"], st["g"].stride(0), lc.LC_F32, 1, wl.beta2)
    torch.cuda.synchronize()
    assert torch.equal(st["theta"], theta1) and torch.equal(st["m"], m1)      # both routes: same bits
    # third route: planes out (the dedicated vote kernel), then apply from planes
    st["theta"].copy_(theta0)
    st["m"].copy_(m0)
    pos = torch.zeros(nw + 8, dtype=torch.int64, device="cuda")
    nzp = torch.zeros(nw + 8, dtype=torch.int64, device="cuda")
    lc.lc_vote_1bit(q, q.stride(0), W, n, pos, nzp, step_no[0], lc.LC_TIE_ZERO)
    lc.lc_apply_update(st["theta"], pos, nzp, n, wl.lr, wl.wd, st["m"], st["m"].stride(0), st["g"], st["g"].stride(0),
                       lc.LC_F32, 1, wl.beta2)
    torch.cuda.synchronize()
    assert torch.equal(st["theta"], theta1) and torch.equal(st["m"], m1)
    assert int(pos[nw:].abs().max()) == 0 and int(nzp[nw:].abs().max()) == 0
    del pos, nzp
    for lo, hi in windows(n, wl.seed):
        words = q[:, lo // 64:(hi + 63) // 64].cpu().numpy().view(np.uint64)
        b = np.stack([orc.unpack_1bit(words[w], hi - lo) for w in range(W)])
        K, S, u = orc.count_sign(b, step_no[0], orc.TIE_ZERO, p=wl.p)
        assert np.array_equal(ksum[lo:hi].cpu().numpy().astype(np.int32), K), "counts in [%d, %d)" % (lo, hi)
        ref_theta = orc.apply(theta0[lo:hi].cpu().numpy(), u, wl.lr, wl.wd)
        assert_close(theta1[lo:hi].cpu().numpy(), ref_theta, "theta in [%d, %d)" % (lo, hi))
        ref_m = orc.momentum(m0[0, lo:hi].cpu().numpy(), st["g"][0, lo:hi].cpu().numpy(), wl.beta2)
        assert_close(m1[0, lo:hi].cpu().numpy(), ref_m, "momentum in [%d, %d)" % (lo, hi))
    # whole range: total of the counts = total population count of the 64 buffers,
    # 0 <= K <= W, and theta moved by -lr * sign(2K - W) after decay
    total_k = int(ksum.to(torch.int64).sum())
    total_pop = int(sum(int(popcount64(q[w, :nw]).sum()) for w in range(W)))
    assert total_k == total_pop
    assert int(ksum.max()) <= W
    u_all = torch.sign(2 * ksum.to(torch.int16) - W).to(torch.float32)
    d = (theta1 - theta0 * (1.0 - wl.lr * wl.wd)) / wl.lr + u_all
    assert float(d.abs().max()) < 1e-2
    # agreement 0.6 with a shared latent sign: few ties, and the vote follows the latent bit
    tie_rate = float((u_all == 0).float().mean())
    assert 0.0 < tie_rate < 0.05


def test_l1_workload():
    """GPT-2-small shapes, 8 workers, L = 15 (the 8-bit L1-quantised allreduce of
    Appendix F.1) as bench.py runs it.  The mean |c| of every worker is compared over
    ALL elements (it must equal the oracle's exactly); levels, sums, theta and momenta on
    sampled windows."""
    wl = synth.workload("l1")
    kernels, st, step_no = bench.build_step(wl, torch, lc, synth)
    n, W, L = wl.n, wl.W, wl.levels
    theta0 = st["theta"].clone()
    m0 = torch.empty((W, n), dtype=torch.float32, device="cuda")
    m0.copy_(st["m"])
    for k in kernels:
        k.fn()
    torch.cuda.synchronize()
    means = st["mean_abs"].cpu().numpy()
    for w in range(W):
        c = orc.local_c(m0[w].cpu().numpy(), st["g"][w].cpu().numpy(), wl.beta1)
        assert orc.mean_abs(c) == means[w], "worker %d: mean |c| over all %d elements" % (w, n)
        del c
    for lo, hi in windows(n, wl.seed):
        mm, gg = host_rows(m0, lo, hi), host_rows(st["g"], lo, hi)
        lev = np.stack([orc.l1_levels(orc.local_c(mm[w], gg[w], wl.beta1), means[w], L) for w in range(W)])
        fields = (lev.astype(np.int16) + L).astype(np.uint8)
        assert np.array_equal(st["q"][:, lo:hi].cpu().numpy(), fields), "level bytes in [%d, %d)" % (lo, hi)
        K, S, u = orc.level_sum_sign(fields, L, step_no[0], orc.TIE_ZERO)
        assert np.array_equal(st["sum_out"][lo:hi].cpu().numpy().astype(np.int32), K)
        assert_close(st["theta"][lo:hi].cpu().numpy(), orc.apply(theta0[lo:hi].cpu().numpy(), u, wl.lr, wl.wd), "theta")
        m_ref = np.stack([orc.momentum(mm[w], gg[w], wl.beta2) for w in range(W)])
        assert_close(host_rows(st["m"], lo, hi), m_ref, "momentum")
    # whole range: the applied update is the sign of (summed bytes - W L)
    K_all = st["sum_out"][:n].to(torch.int16)
    u_all = torch.sign(K_all - W * L).to(torch.float32)
    d = (st["theta"] - theta0 * (1.0 - wl.lr * wl.wd)) / wl.lr + u_all
    assert float(d.abs().max()) < 1e-2 and int(K_all.max()) <= 2 * L * W
    assert int(st["q"][:, :n].max()) <= 2 * L


def test_l1_workload_per_tensor_scales():
    """The same workload with one scale, rate and decay per tensor through the group-table
    calls (bench.py --groups): every one of the 148 x 8 means is compared over all of its
    elements, levels, sums and theta on sampled windows against the oracle applied tensor by
    tensor."""
    wl = synth.workload("l1")
    kernels, st, step_no = bench.build_step(wl, torch, lc, synth, groups=True)
    n, W, L = wl.n, wl.W, wl.levels
    theta0 = st["theta"].clone()
    m0 = torch.empty((W, n), dtype=torch.float32, device="cuda")
    m0.copy_(st["m"])
    for k in kernels:
        k.fn()
    torch.cuda.synchronize()
    ends = (st["end64"].cpu().numpy().astype(np.int64) * 64).tolist()
    starts = [0] + ends[:-1]
    assert ends[-1] == n and len(ends) == len(wl.tensors)
    means = st["mean_abs"].cpu().numpy()
    lr_t, wd_t = st["lr_t"].cpu().numpy(), st["wd_t"].cpu().numpy()
    for w in range(W):
        c = orc.local_c(m0[w].cpu().numpy(), st["g"][w].cpu().numpy(), wl.beta1)
        for s, (lo, hi) in enumerate(zip(starts, ends)):
            assert orc.mean_abs(c[lo:hi]) == means[w, s], "worker %d, tensor %s" % (w, wl.tensors[s][0])
        del c
    # windows: the sampled ones plus one around every 16th tensor boundary
    spans = windows(n, wl.seed) + [(max(0, e - 2048), min(n, e + 2048)) for e in ends[::16]]
    for lo, hi in spans:
        mm, gg = host_rows(m0, lo, hi), host_rows(st["g"], lo, hi)
        seg = np.searchsorted(np.asarray(ends), np.arange(lo, hi), side="right")
        fields = np.empty((W, hi - lo), np.uint8)
        theta_ref = theta0[lo:hi].cpu().numpy().copy()
        for s in np.unique(seg):
            sel = np.flatnonzero(seg == s)
            a, b = int(sel[0]), int(sel[-1]) + 1
            for w in range(W):
                lev = orc.l1_levels(orc.local_c(mm[w, a:b], gg[w, a:b], wl.beta1), means[w, s], L)
                fields[w, a:b] = (lev.astype(np.int16) + L).astype(np.uint8)
            K, S, u = orc.level_sum_sign(fields[:, a:b], L, step_no[0], orc.TIE_ZERO)
            assert np.array_equal(st["sum_out"][lo + a:lo + b].cpu().numpy().astype(np.int32), K)
            theta_ref[a:b] = orc.apply(theta_ref[a:b], u, float(lr_t[s]), float(wd_t[s]))
        assert np.array_equal(st["q"][:, lo:hi].cpu().numpy(), fields), "level bytes in [%d, %d)" % (lo, hi)
        assert_close(st["theta"][lo:hi].cpu().numpy(), theta_ref, "theta in [%d, %d)" % (lo, hi))
    assert int(st["q"][:, :n].max()) <= 2 * L and int(st["sum_out"][:n].max()) <= 2 * L * W


def test_ternary_workload():
    """GPT-2-small shapes, 8 workers, the two-plane ternary wire format of Appendix B.1 as
    bench.py runs it: planes, theta and momenta on sampled windows, and over the whole
    range the applied update against the planes' own counts."""
    wl = synth.workload("t2")
    kernels, st, step_no = bench.build_step(wl, torch, lc, synth)
    n, W = wl.n, wl.W
    nw = (n + 63) // 64
    theta0 = st["theta"].clone()
    m0 = torch.empty((W, n), dtype=torch.float32, device="cuda")
    m0.copy_(st["m"])
    for k in kernels:
        k.fn()
    torch.cuda.synchronize()
    hp = dict(beta1=wl.beta1, beta2=wl.beta2, lr=wl.lr, wd=wl.wd)
    for lo, hi in windows(n, wl.seed):
        ref = orc.step_ternary(theta0[lo:hi].cpu().numpy(), host_rows(m0, lo, hi), host_rows(st["g"], lo, hi), **hp)
        w0, w1 = lo // 64, (hi + 63) // 64
        assert np.array_equal(st["pos"][:, w0:w1].cpu().numpy().view(np.uint64), ref["pos_w"]), "pos planes in [%d, %d)" % (lo, hi)
        assert np.array_equal(st["nz"][:, w0:w1].cpu().numpy().view(np.uint64), ref["nz_w"]), "nz planes in [%d, %d)" % (lo, hi)
        assert_close(st["theta"][lo:hi].cpu().numpy(), ref["theta"], "theta in [%d, %d)" % (lo, hi))
        assert_close(host_rows(st["m"], lo, hi), ref["m"], "momentum in [%d, %d)" % (lo, hi))
    # whole range: K+ and K- from population counts of the planes, per 64-element word:
    # sum over the word of u = sum of sign(K+ - K-) cannot be checked per element cheaply,
    # but unanimous words can: all workers pos on every bit -> every u = +1, no worker nz -> u = 0
    pos, nz = st["pos"][:, :nw], st["nz"][:, :nw]
    all_pos, any_nz = pos[0] & nz[0], nz[0].clone()
    for w in range(1, W):
        all_pos &= pos[w] & nz[w]
        any_nz |= nz[w]
    d = (st["theta"] - theta0 * (1.0 - wl.lr * wl.wd)) / wl.lr            # = -u up to rounding
    assert float((d - d.round()).abs().max()) < 1e-2 and float(d.abs().max()) < 1.01
    u_all = -d.round()
    shifts = torch.arange(64, device="cuda", dtype=torch.int64)
    for lo in range(0, nw, 1 << 22):
        hi = min(nw, lo + (1 << 22))
        count = min(n, hi * 64) - lo * 64
        a = ((all_pos[lo:hi, None] >> shifts) & 1).view(-1)[:count].bool()
        z = ((any_nz[lo:hi, None] >> shifts) & 1).view(-1)[:count].bool()
        uu = u_all[lo * 64: lo * 64 + count]
        assert bool((uu[a] == 1).all()) and bool((uu[~z] == 0).all())
