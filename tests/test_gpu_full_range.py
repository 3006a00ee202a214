"""Full-range parity: the five benchmark workloads, run exactly as bench.py runs them (same
buffers, same C-ABI calls, same launch configuration), compared with the CPU oracle element
by element over the WHOLE range -- every packed word, field and count bit for bit, every
parameter and momentum within 1e-6 relative / 1e-7 absolute.  The range is cut into chunks;
each chunk's inputs and outputs come to the host, the oracle runs on the chunk, and a pool
of host threads works through the chunks (the oracle's C loops release the interpreter
lock).  The sampled-window tests of test_gpu_full_size.py remain the fast tier."""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import bench
import oracle as orc
import paper_2411_16462_amd as lc
from harness import ATOL, RTOL, g_host
from paper_2411_16462_amd import synth

pytestmark = pytest.mark.gpu

CHUNK = 1 << 22                                   # elements per chunk (a multiple of 64)
THREADS = min(16, len(os.sched_getaffinity(0)))   # one GPU's share of the box


def spans(n, part=0, parts=1):
    """64-aligned chunks of [0, n); part / parts selects a contiguous share of them."""
    all_spans = [(lo, min(n, lo + CHUNK)) for lo in range(0, n, CHUNK)]
    per = (len(all_spans) + parts - 1) // parts
    return all_spans[part * per:(part + 1) * per]


def worst_excess(got, ref):
    return float((np.abs(got.astype(np.float64) - ref) - (ATOL + RTOL * np.abs(ref))).max())


def over_chunks(fn, chunk_list):
    """fn(lo, hi) -> (number of elements compared, number of ties); raises on a mismatch"""
    with ThreadPoolExecutor(max_workers=THREADS) as ex:
        out = list(ex.map(lambda s: fn(*s), chunk_list))
    return sum(a for a, _ in out), sum(b for _, b in out)


def clone_rows(t):
    out = torch.empty(t.shape, dtype=t.dtype, device=t.device)
    out.copy_(t)
    return out


@pytest.mark.parametrize("name,part,parts", [("c0", 0, 1), ("c1", 0, 1), ("c2", 0, 1),
                                              ("c3", 0, 3), ("c3", 1, 3), ("c3", 2, 3)])
def test_training_workload_every_element(name, part, parts):
    wl = synth.workload(name)
    kernels, st, step_no = bench.build_step(wl, torch, lc, synth)
    n, W = wl.n, wl.W
    theta0, m0 = st["theta"].clone(), clone_rows(st["m"])
    for k in kernels:
        k.fn()
    torch.cuda.synchronize()
    gd = orc.BF16 if wl.g_dtype == "bf16" else orc.F32
    hp = dict(beta1=wl.beta1, beta2=wl.beta2, lr=wl.lr, wd=wl.wd, step=step_no[0], g_dtype=gd)
    C = lc.lc_container_bits(wl.p)

    def check(lo, hi):
        th, mm = theta0[lo:hi].cpu().numpy(), m0[:, lo:hi].cpu().numpy()
        gg = g_host(st["g"][:, lo:hi])
        where = "%s [%d, %d)" % (name, lo, hi)
        if wl.mode == "1bit":
            ref = orc.step_1bit(th, mm, gg, **hp)
            got = st["q"][:, lo // 64:(hi + 63) // 64].cpu().numpy().view(np.uint64)
            assert np.array_equal(got, ref["words"]), "packed words, " + where
        else:
            ref = orc.step_pbit(th, mm, gg, p=wl.p, **hp)
            b0, b1 = lo * C // 8, (hi * C + 7) // 8
            assert np.array_equal(st["q"][:, b0:b1].cpu().numpy(), ref["fields"]), "fields, " + where
            assert np.array_equal(st["sum_out"][b0:b1].cpu().numpy(), ref["sum_fields"]), "field sums, " + where
        assert worst_excess(st["theta"][lo:hi].cpu().numpy(), ref["theta"]) <= 0.0, "theta, " + where
        m_ref = ref["m"]
        if wl.momentum_avg:
            m_ref = np.broadcast_to(orc.momentum_avg(m_ref.astype(np.float32)), m_ref.shape)
        assert worst_excess(st["m"][:, lo:hi].cpu().numpy(), m_ref) <= 0.0, "momentum, " + where
        return hi - lo, int((ref["u"] == 0).sum())

    chunk_list = spans(n, part, parts)
    done, ties = over_chunks(check, chunk_list)
    assert done == chunk_list[-1][1] - chunk_list[0][0]
    if W % 2 == 0:
        assert ties > 0          # the tie rule was exercised


@pytest.mark.parametrize("part,parts", [(0, 4), (1, 4), (2, 4), (3, 4)])
def test_reduction_only_workload_every_element(part, parts):
    """N = 1.3e9, 64 pre-packed rows: the fused majority vote + apply, and the p = 7 sum of
    signs with its byte counts, both against the oracle on every element of the part."""
    wl = synth.workload("c4")
    kernels, st, step_no = bench.build_step(wl, torch, lc, synth)
    n, W = wl.n, wl.W
    q = st["q"]
    theta0, m0 = st["theta"].clone(), st["m"].clone()
    for k in kernels:
        k.fn()
    torch.cuda.synchronize()
    theta1, m1 = st["theta"].clone(), st["m"].clone()
    st["theta"].copy_(theta0)
    st["m"].copy_(m0)
    ksum = torch.zeros(n, dtype=torch.uint8, device="cuda")
    lc.lc_pbit_sum_apply(q, q.stride(0) * 8, 1, W, n, wl.p, ksum, step_no[0], lc.LC_TIE_ZERO, st["theta"], wl.lr, wl.wd,
                         st["m"], st["m"].stride(0), st["g"], st["g"].stride(0), lc.LC_F32, 1, wl.beta2)
    torch.cuda.synchronize()

    def check(lo, hi):
        where = "c4 [%d, %d)" % (lo, hi)
        words = q[:, lo // 64:(hi + 63) // 64].cpu().numpy().view(np.uint64)
        b = np.stack([orc.unpack_1bit(words[w], hi - lo) for w in range(W)])
        K, S, u = orc.count_sign(b, step_no[0], orc.TIE_ZERO, p=wl.p)
        del b
        assert np.array_equal(ksum[lo:hi].cpu().numpy().astype(np.int32), K), "counts, " + where
        ref_theta = orc.apply(theta0[lo:hi].cpu().numpy(), u, wl.lr, wl.wd)
        ref_m = orc.momentum(m0[0, lo:hi].cpu().numpy(), st["g"][0, lo:hi].cpu().numpy(), wl.beta2)
        for label, th, mm in (("vote", theta1, m1), ("sum", st["theta"], st["m"])):
            assert worst_excess(th[lo:hi].cpu().numpy(), ref_theta) <= 0.0, "theta (%s), %s" % (label, where)
            assert worst_excess(mm[0, lo:hi].cpu().numpy(), ref_m) <= 0.0, "momentum (%s), %s" % (label, where)
        return hi - lo, int((u == 0).sum())

    chunk_list = spans(n, part, parts)
    done, ties = over_chunks(check, chunk_list)
    assert done == chunk_list[-1][1] - chunk_list[0][0]
    assert ties > 0


def test_ternary_workload_every_element():
    """GPT-2-small shapes, 8 workers, the two-plane ternary wire format of Appendix B.1."""
    wl = synth.workload("t2")
    kernels, st, step_no = bench.build_step(wl, torch, lc, synth)
    n, W = wl.n, wl.W
    theta0, m0 = st["theta"].clone(), clone_rows(st["m"])
    for k in kernels:
        k.fn()
    torch.cuda.synchronize()
    hp = dict(beta1=wl.beta1, beta2=wl.beta2, lr=wl.lr, wd=wl.wd)

    def check(lo, hi):
        where = "t2 [%d, %d)" % (lo, hi)
        ref = orc.step_ternary(theta0[lo:hi].cpu().numpy(), m0[:, lo:hi].cpu().numpy(), st["g"][:, lo:hi].cpu().numpy(), **hp)
        w0, w1 = lo // 64, (hi + 63) // 64
        assert np.array_equal(st["pos"][:, w0:w1].cpu().numpy().view(np.uint64), ref["pos_w"]), "pos planes, " + where
        assert np.array_equal(st["nz"][:, w0:w1].cpu().numpy().view(np.uint64), ref["nz_w"]), "nz planes, " + where
        assert worst_excess(st["theta"][lo:hi].cpu().numpy(), ref["theta"]) <= 0.0, "theta, " + where
        assert worst_excess(st["m"][:, lo:hi].cpu().numpy(), ref["m"]) <= 0.0, "momentum, " + where
        return hi - lo, int((ref["u"] == 0).sum())

    done, zeros = over_chunks(check, spans(n))
    assert done == n and zeros > 0


def test_l1_workload_every_element():
    """GPT-2-small shapes, 8 workers, L = 15 (the 8-bit L1-quantised allreduce of Appendix
    F.1): the exact means over all elements, then every level byte, level sum, parameter and
    momentum."""
    wl = synth.workload("l1")
    kernels, st, step_no = bench.build_step(wl, torch, lc, synth)
    n, W, L = wl.n, wl.W, wl.levels
    theta0, m0 = st["theta"].clone(), clone_rows(st["m"])
    for k in kernels:
        k.fn()
    torch.cuda.synchronize()
    means = st["mean_abs"].cpu().numpy()

    def mean_of(w):
        c = orc.local_c(m0[w].cpu().numpy(), st["g"][w].cpu().numpy(), wl.beta1)
        return orc.mean_abs(c)

    with ThreadPoolExecutor(max_workers=min(W, THREADS)) as ex:
        want = list(ex.map(mean_of, range(W)))
    assert means.tolist() == want, "mean |c| over all elements"

    def check(lo, hi):
        where = "l1 [%d, %d)" % (lo, hi)
        mm, gg = m0[:, lo:hi].cpu().numpy(), st["g"][:, lo:hi].cpu().numpy()
        lev = np.stack([orc.l1_levels(orc.local_c(mm[w], gg[w], wl.beta1), means[w], L) for w in range(W)])
        fields = (lev.astype(np.int16) + L).astype(np.uint8)
        assert np.array_equal(st["q"][:, lo:hi].cpu().numpy(), fields), "level bytes, " + where
        K, S, u = orc.level_sum_sign(fields, L, step_no[0], orc.TIE_ZERO)
        assert np.array_equal(st["sum_out"][lo:hi].cpu().numpy().astype(np.int32), K), "level sums, " + where
        ref_theta = orc.apply(theta0[lo:hi].cpu().numpy(), u, wl.lr, wl.wd)
        assert worst_excess(st["theta"][lo:hi].cpu().numpy(), ref_theta) <= 0.0, "theta, " + where
        m_ref = np.stack([orc.momentum(mm[w], gg[w], wl.beta2) for w in range(W)])
        assert worst_excess(st["m"][:, lo:hi].cpu().numpy(), m_ref) <= 0.0, "momentum, " + where
        return hi - lo, int((u == 0).sum())

    done, ties = over_chunks(check, spans(n))
    assert done == n and ties > 0
