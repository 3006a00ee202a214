"""Randomised differential test: many seeded random configurations (sizes, worker counts,
rules, dtypes, hyper-parameters, input regimes) through every path of the library,
each against the oracle.  Deterministic: the configurations come from one fixed seed.
For a longer campaign LIONCUB_RANDOM_SCALE multiplies the number of configurations and
LIONCUB_RANDOM_SEED shifts the seeds (both default to the committed set)."""
import os

import numpy as np
import pytest
import torch

import oracle as orc
import paper_2411_16462_amd as lc
from harness import Case, assert_close, guarded, hip_update_pack, oracle_step, untouched, words_of

pytestmark = pytest.mark.gpu


def configs(count, seed):
    count *= int(os.environ.get("LIONCUB_RANDOM_SCALE", "1"))
    rng = np.random.default_rng(seed + int(os.environ.get("LIONCUB_RANDOM_SEED", "0")))
    out = []
    for i in range(count):
        n = int(rng.choice([rng.integers(1, 300), rng.integers(300, 5000), rng.integers(5000, 70000)]))
        out.append(dict(
            i=i, n=n, W=int(rng.choice([1, 2, 3, 4, 5, 7, 8, 9, 12, 15, 16, 31, 32, 33, 64, 100])),
            g_dtype=str(rng.choice(["f32", "bf16"])), step=int(rng.integers(1, 1000)),
            zero=int(rng.integers(0, 3)), tie=int(rng.integers(0, 2)),
            beta1=float(rng.choice([0.0, 0.5, 0.8, 0.9, 0.95, 1.0])), beta2=float(rng.choice([0.0, 0.9, 0.95, 0.99, 1.0])),
            lr=float(rng.choice([0.0, 1e-5, 1e-4, 3e-3])), wd=float(rng.choice([0.0, 1e-2, 0.1, 1.0])),
            regime=str(rng.choice(["shared_m", "no_m", "sparse", "tiny"])), seed=int(rng.integers(1 << 30))))
    return out


def make_case(c):
    kw = dict(m_scale=0.0) if c["regime"] in ("no_m", "sparse") else dict(m_spread=0.5)
    case = Case(c["n"], c["W"], seed=c["seed"], g_dtype=c["g_dtype"], **kw)
    if c["regime"] == "sparse":
        mask = torch.rand(case.g.shape, device="cuda", generator=torch.Generator(device="cuda").manual_seed(c["seed"])) < 0.5
        case.g[mask] = 0
    if c["regime"] == "tiny":
        case.g.mul_(1e-30)
        case.m.mul_(1e-30)
    case.snapshot()
    return case


@pytest.mark.parametrize("c", configs(40, 20241127), ids=lambda c: "cfg%d" % c["i"])
def test_random_1bit_and_pbit(c):
    hp = dict(beta1=c["beta1"], beta2=c["beta2"], lr=c["lr"], wd=c["wd"])
    n, W, step = c["n"], c["W"], c["step"]
    nw = (n + 63) // 64
    ogd = orc.BF16 if c["g_dtype"] == "bf16" else orc.F32
    # 1-bit path, fused vote + apply
    case = make_case(c)
    ref = orc.step_1bit(case.theta0, case.m0, case.g0, step=step, zero=c["zero"], tie=c["tie"], g_dtype=ogd, **hp)
    q, nbytes = hip_update_pack(case, hp, step, 1, c["zero"])
    lc.lc_vote_apply_1bit(q, q.stride(0) // 8, W, n, step, c["tie"], case.theta, hp["lr"], hp["wd"], None, 0, None, 0,
                          lc.LC_F32, 0, hp["beta2"])
    torch.cuda.synchronize()
    assert np.array_equal(words_of(q, nw), ref["words"]) and untouched(q, nbytes)
    assert_close(case.theta.cpu().numpy(), ref["theta"], "theta")
    assert_close(case.m.cpu().numpy(), ref["m"], "momentum")
    # p-bit path with the smallest p that serves W workers
    p = max(1, int(W).bit_length())
    if p <= 8:
        C = lc.lc_container_bits(p)
        case = make_case(c)
        ref = orc.step_pbit(case.theta0, case.m0, case.g0, p=p, step=step, zero=c["zero"], tie=c["tie"], g_dtype=ogd, **hp)
        q, nbytes = hip_update_pack(case, hp, step, C, c["zero"])
        fb = nw * 8 if C == 1 else (n * C + 7) // 8
        ksum = guarded(1, fb, "cuda")
        lc.lc_pbit_sum_apply(q, q.stride(0), C, W, n, p, ksum, step, c["tie"], case.theta, hp["lr"], hp["wd"], None, 0, None,
                             0, lc.LC_F32, 0, hp["beta2"])
        torch.cuda.synchronize()
        assert np.array_equal(ksum[0, :(n * C + 7) // 8].cpu().numpy(), ref["sum_fields"]) and untouched(ksum, fb)
        assert_close(case.theta.cpu().numpy(), ref["theta"], "theta (p-bit)")


@pytest.mark.parametrize("c", configs(24, 777), ids=lambda c: "cfg%d" % c["i"])
def test_random_ternary_and_l1(c):
    hp = dict(beta1=c["beta1"], beta2=c["beta2"], lr=c["lr"], wd=c["wd"])
    n, W = c["n"], c["W"]
    nw = (n + 63) // 64
    ogd = orc.BF16 if c["g_dtype"] == "bf16" else orc.F32
    case = make_case(c)
    ref = orc.step_ternary(case.theta0, case.m0, case.g0, g_dtype=ogd, **hp)
    pos, nz = guarded(W, nw * 8, "cuda"), guarded(W, nw * 8, "cuda")
    lc.lc_local_update_pack_ternary(case.g, case.g.stride(0), case.gd, case.m, case.m.stride(0), W, n, hp["beta1"], 1,
                                    hp["beta2"], pos, nz, pos.stride(0) // 8)
    lc.lc_vote_apply_ternary(pos, nz, pos.stride(0) // 8, W, n, case.theta, hp["lr"], hp["wd"], None, 0, None, 0, lc.LC_F32,
                             0, hp["beta2"])
    torch.cuda.synchronize()
    assert np.array_equal(words_of(pos, nw), ref["pos_w"]) and np.array_equal(words_of(nz, nw), ref["nz_w"])
    assert_close(case.theta.cpu().numpy(), ref["theta"], "theta (ternary)")
    L = min(127, 255 // (2 * W))
    if L >= 1:
        case = make_case(c)
        ref = orc.step_l1(case.theta0, case.m0, case.g0, L=L, step=c["step"], tie=c["tie"], g_dtype=ogd, **hp)
        mean = torch.zeros(W, dtype=torch.float64, device="cuda")
        ws = torch.zeros(W * lc.LC_L1_WORKSPACE_WORDS, dtype=torch.int64, device="cuda")
        lc.lc_l1_mean_abs(case.g, case.g.stride(0), case.gd, case.m, case.m.stride(0), W, n, hp["beta1"], mean, ws)
        lv = guarded(W, n, "cuda")
        lc.lc_l1_quantize_pack(case.g, case.g.stride(0), case.gd, case.m, case.m.stride(0), W, n, hp["beta1"], 1, hp["beta2"],
                               L, mean, lv, lv.stride(0))
        lc.lc_level_sum_apply(lv, lv.stride(0), W, n, L, None, c["step"], c["tie"], case.theta, hp["lr"], hp["wd"], None, 0,
                              None, 0, lc.LC_F32, 0, hp["beta2"])
        torch.cuda.synchronize()
        assert np.array_equal(mean.cpu().numpy(), ref["mean_abs"])
        assert np.array_equal(lv[:, :n].cpu().numpy(), ref["fields"]) and untouched(lv, n)
        assert_close(case.theta.cpu().numpy(), ref["theta"], "theta (L1)")
        assert_close(case.m.cpu().numpy(), ref["m"], "momentum (L1)")


def random_table(n, rng):
    """A random group table over n elements: ascending ends in units of 64 elements, with
    repeated ends (empty segments) now and then; the last end reaches n."""
    n64 = (n + 63) // 64
    G = int(rng.integers(1, 12))
    ends = sorted(int(v) for v in rng.integers(0, n64 + 1, G - 1)) + [n64]
    bounds = [0] + [min(e * 64, n) for e in ends]
    return ends, bounds


@pytest.mark.parametrize("c", configs(32, 31337), ids=lambda c: "cfg%d" % c["i"])
def test_random_routes_agree(c):
    """Every route to the same update gives the same bits, and all match the oracle: fused
    vote+apply; vote to planes, then apply from planes (with the momentum update moved into
    the apply); the counts K from 1-bit rows through the p-bit call; and one launch with a
    random per-group table against the oracle applied segment by segment."""
    hp = dict(beta1=c["beta1"], beta2=c["beta2"], lr=c["lr"], wd=c["wd"])
    n, W, step, tie = c["n"], c["W"], c["step"], c["tie"]
    nw = (n + 63) // 64
    ogd = orc.BF16 if c["g_dtype"] == "bf16" else orc.F32
    rng = np.random.default_rng(c["seed"])
    a, b, d = make_case(c), make_case(c), make_case(c)
    ref = orc.step_1bit(a.theta0, a.m0, a.g0, step=step, zero=c["zero"], tie=tie, g_dtype=ogd, **hp)
    # route A: update+pack with the momentum update, fused vote+apply
    qa, nbytes = hip_update_pack(a, hp, step, 1, c["zero"])
    lc.lc_vote_apply_1bit(qa, qa.stride(0) // 8, W, n, step, tie, a.theta, hp["lr"], hp["wd"], None, 0, None, 0, lc.LC_F32, 0,
                          hp["beta2"])
    # route B: pack without touching m, planes out, apply from planes with all W momentum rows
    qb, _ = hip_update_pack(b, hp, step, 1, c["zero"], update_m=False)
    pos, nz = guarded(1, nw * 8, "cuda"), guarded(1, nw * 8, "cuda")
    lc.lc_vote_1bit(qb, qb.stride(0) // 8, W, n, pos, nz, step, tie)
    lc.lc_apply_update(b.theta, pos, nz, n, hp["lr"], hp["wd"], b.m, b.m.stride(0), b.g, b.g.stride(0), b.gd, W, hp["beta2"])
    torch.cuda.synchronize()
    assert torch.equal(qa, qb)
    assert np.array_equal(words_of(pos, nw)[0], ref["pos"]) and np.array_equal(words_of(nz, nw)[0], ref["nz"])
    assert untouched(pos, nw * 8) and untouched(nz, nw * 8)
    assert torch.equal(a.theta, b.theta) and torch.equal(a.m, b.m)
    assert_close(a.theta.cpu().numpy(), ref["theta"], "theta")
    assert_close(a.m.cpu().numpy(), ref["m"], "momentum")
    # route C: the counts K from the same 1-bit rows through the p-bit call (momentum fused in)
    p = max(2, int(W).bit_length())
    if p <= 8:
        C = lc.lc_container_bits(p)
        ksum = guarded(1, (n * C + 7) // 8, "cuda")
        qd, _ = hip_update_pack(d, hp, step, 1, c["zero"], update_m=False)
        lc.lc_pbit_sum_apply(qd, qd.stride(0), 1, W, n, p, ksum, step, tie, d.theta, hp["lr"], hp["wd"], d.m, d.m.stride(0),
                             d.g, d.g.stride(0), d.gd, W, hp["beta2"])
        torch.cuda.synchronize()
        rp = orc.step_pbit(d.theta0, d.m0, d.g0, p=p, step=step, zero=c["zero"], tie=tie, g_dtype=ogd, **hp)
        assert np.array_equal(ksum[0, :(n * C + 7) // 8].cpu().numpy(), rp["sum_fields"]) and untouched(ksum, (n * C + 7) // 8)
        assert torch.equal(d.theta, a.theta) and torch.equal(d.m, a.m)
    # route D: a random group table in one launch (no momentum streams), on fresh parameters
    ends, bounds = random_table(n, rng)
    G = len(ends)
    lrs = [float(v) for v in rng.choice([0.0, 1e-5, 1e-4, 3e-3, 3e-2], G)]
    wds = [float(v) for v in rng.choice([0.0, 1e-2, 0.1, 1.0], G)]
    e = make_case(c)
    end_t = torch.tensor(ends, dtype=torch.int32, device="cuda")
    lr_t = torch.tensor(lrs, dtype=torch.float32, device="cuda")
    wd_t = torch.tensor(wds, dtype=torch.float32, device="cuda")
    lc.lc_vote_apply_1bit_groups(qa, qa.stride(0) // 8, W, n, step, tie, e.theta, end_t, lr_t, wd_t, G)
    torch.cuda.synchronize()
    want = np.empty(n, np.float64)
    for s in range(G):
        lo, hi = bounds[s], bounds[s + 1]
        want[lo:hi] = orc.apply(e.theta0[lo:hi], ref["u"][lo:hi], lrs[s], wds[s])
    assert_close(e.theta.cpu().numpy(), want, "theta with a random group table")
