"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs -- bit-exact for signs, packed words, fields, counts and votes; within
1e-6 relative / 1e-7 absolute for updated parameters and momenta."""
import numpy as np
import pytest
import torch

import oracle as orc
import paper_2411_16462_amd as lc
from harness import (SENTINEL, Case, assert_close, clone_rows, guarded, hip_update_pack, oracle_step, untouched, words_of)

pytestmark = pytest.mark.gpu

HP = dict(beta1=0.9, beta2=0.99, lr=1e-4, wd=0.1)
SIZES = [1, 63, 64, 65, 1000, 1023, 1024, 1025, 4095, 4096, 4097, 16384 + 17, 3 * 16384]


def nwords(n):
    return (n + 63) // 64


def run_1bit(case, step, zero=lc.LC_ZERO_ALT, tie=lc.LC_TIE_ZERO, fused=True, hp=HP):
    """update+pack, then vote (+apply).  Returns every stage as numpy."""
    n, W = case.n, case.W
    nw = nwords(n)
    q, nbytes = hip_update_pack(case, hp, step, 1, zero)
    out = dict(words=words_of(q, nw), q_clean=untouched(q, nbytes), m=case.m.cpu().numpy())
    pos = guarded(1, nw * 8, case.device)
    nz = guarded(1, nw * 8, case.device)
    lc.lc_vote_1bit(q, q.stride(0) // 8, W, n, pos, nz, step, tie)
    out["pos"], out["nz"] = words_of(pos, nw)[0], words_of(nz, nw)[0]
    out["planes_clean"] = untouched(pos, nw * 8) and untouched(nz, nw * 8)
    if fused:
        lc.lc_vote_apply_1bit(q, q.stride(0) // 8, W, n, step, tie, case.theta, hp["lr"], hp["wd"], None, 0, None, 0,
                              lc.LC_F32, 0, hp["beta2"])
    else:
        lc.lc_apply_update(case.theta, pos, nz, n, hp["lr"], hp["wd"], None, 0, None, 0, lc.LC_F32, 0, hp["beta2"])
    torch.cuda.synchronize()
    out["theta"] = case.theta.cpu().numpy()
    return out


def check_1bit(out, ref):
    assert np.array_equal(out["words"], ref["words"]), "packed sign words"
    assert out["q_clean"] and out["planes_clean"], "wrote past the end of a packed row"
    assert np.array_equal(out["pos"], ref["pos"]), "vote plane pos"
    assert np.array_equal(out["nz"], ref["nz"]), "vote plane nz"
    assert_close(out["m"], ref["m"], "momentum")
    assert_close(out["theta"], ref["theta"], "theta")


@pytest.mark.parametrize("n", SIZES)
@pytest.mark.parametrize("W", [1, 4, 7])
def test_1bit_sizes(n, W):
    for step, fused in ((1, True), (2, False)):
        case = Case(n, W, seed=1000 + n + W, m_spread=1.0)
        out = run_1bit(case, step, fused=fused)
        check_1bit(out, oracle_step(case, HP, step))


@pytest.mark.parametrize("W", [2, 3, 8, 9, 15, 16, 17, 31, 64, 65, 127, 128, 255])
def test_1bit_worker_counts(W):
    n = 4096 + 333
    case = Case(n, W, seed=2000 + W, m_scale=0.0)          # m = 0: signs nearly independent -> many ties
    out = run_1bit(case, step=1)
    ref = oracle_step(case, HP, 1)
    check_1bit(out, ref)
    if W % 2 == 0 and W <= 16:
        assert (ref["u"] == 0).mean() > 0.05                # ties really occur in this case


@pytest.mark.parametrize("g_dtype", ["f32", "bf16"])
@pytest.mark.parametrize("zero", [lc.LC_ZERO_ALT, lc.LC_ZERO_POS, lc.LC_ZERO_NEG])
@pytest.mark.parametrize("tie", [lc.LC_TIE_ZERO, lc.LC_TIE_ALT])
@pytest.mark.parametrize("step", [1, 2])
def test_1bit_rules_and_dtypes(g_dtype, zero, tie, step):
    n, W = 20000, 4
    case = Case(n, W, seed=3000, g_dtype=g_dtype, m_scale=0.0)
    # exact zeros of c: whole columns (all workers) and single workers
    case.g[:, 100:300] = 0
    case.g[1, 5000:5100] = 0
    case.g[:, n - 7:] = 0
    case.snapshot()
    out = run_1bit(case, step, zero, tie)
    ref = oracle_step(case, HP, step, zero, tie)
    assert (ref["s"][:, 100:300] == 0).all()
    check_1bit(out, ref)


@pytest.mark.parametrize("p,W", [(2, 2), (4, 8), (8, 6)])
@pytest.mark.parametrize("zero", [lc.LC_ZERO_ALT, lc.LC_ZERO_POS, lc.LC_ZERO_NEG])
@pytest.mark.parametrize("tie", [lc.LC_TIE_ZERO, lc.LC_TIE_ALT])
@pytest.mark.parametrize("step", [1, 2])
def test_pbit_rules(p, W, zero, tie, step):
    """Every zero rule and tie rule on odd and even iterations through the field path: exact
    zeros of c in whole columns and for single workers, an even worker count so that ties occur."""
    n = 12345
    C = lc.lc_container_bits(p)
    case = Case(n, W, seed=3100 + p, m_scale=0.0)
    case.g[:, 100:300] = 0
    case.g[1, 5000:5100] = 0
    case.g[:, n - 7:] = 0
    case.snapshot()
    ref = oracle_step(case, HP, step, zero, tie, p=p)
    assert (ref["s"][:, 100:300] == 0).all() and (ref["S"] == 0).any()
    q, nbytes = hip_update_pack(case, HP, step, C, zero)
    assert np.array_equal(q[:, :nbytes].cpu().numpy(), ref["fields"]), "p-bit fields"
    nw, fb = nwords(n), (n * C + 7) // 8
    sum_out = guarded(1, fb, case.device)
    pos, nz = guarded(1, nw * 8, case.device), guarded(1, nw * 8, case.device)
    lc.lc_pbit_sum_sign(q, q.stride(0), C, W, n, p, sum_out, pos, nz, step, tie)
    lc.lc_pbit_sum_apply(q, q.stride(0), C, W, n, p, None, step, tie, case.theta, HP["lr"], HP["wd"], None, 0, None, 0,
                         lc.LC_F32, 0, HP["beta2"])
    torch.cuda.synchronize()
    assert np.array_equal(sum_out[0, :fb].cpu().numpy(), ref["sum_fields"]), "field sums"
    assert np.array_equal(words_of(pos, nw)[0], ref["pos"]) and np.array_equal(words_of(nz, nw)[0], ref["nz"])
    assert_close(case.theta.cpu().numpy(), ref["theta"], "theta")


def test_special_values():
    """NaN, infinities, signed zeros, denormals and exact cancellation in c."""
    n, W = 4096 + 64, 3
    case = Case(n, W, seed=4000)
    tiny = 2.0 ** -148
    vals_m = torch.tensor([0.0, -0.0, float("nan"), float("inf"), -float("inf"), tiny, -tiny, 1.0, 1e-38, -1e-38])
    vals_g = torch.tensor([0.0, -0.0, 1.0, 1.0, 1.0, 0.0, 0.0, -9.0, -1e-38, 1e-38])
    k = vals_m.numel()
    for base in (0, 4096):                     # once in the vector path, once in the ragged tail
        case.m[:, base:base + k] = vals_m.to(case.m.device)
        case.g[:, base:base + k] = vals_g.to(case.g.device)
    case.snapshot()
    hp = dict(HP, beta1=0.5)
    n_w = nwords(n)
    for step in (1, 2):
        q, nbytes = hip_update_pack(case, hp, step, 1, update_m=False)
        ref = oracle_step(case, hp, step)
        assert ref["s"][0, :8].tolist() == [0, 0, 0, 1, -1, 1, -1, -1]
        assert np.array_equal(words_of(q, n_w), ref["words"])


def test_update_without_q_and_pack_without_update():
    n, W = 10000, 3
    case = Case(n, W, seed=5000)
    ref = oracle_step(case, HP, 1)
    q, nbytes = hip_update_pack(case, HP, 1, 1, update_m=False)
    assert np.array_equal(words_of(q, nwords(n)), ref["words"])
    assert np.array_equal(case.m.cpu().numpy(), case.m0)          # momentum untouched
    hip_update_pack(case, HP, 1, 1, want_q=False)
    assert_close(case.m.cpu().numpy(), ref["m"], "momentum")


@pytest.mark.parametrize("p,W", [(1, 1), (2, 3), (3, 7), (4, 8), (4, 15), (5, 16), (7, 64), (8, 125), (8, 255)])
@pytest.mark.parametrize("n", [1, 31, 1000, 2048 + 5, 4096, 16384 + 17])
def test_pbit_fields(p, W, n):
    C = lc.lc_container_bits(p)
    step = 1 + (n % 2)
    case = Case(n, W, seed=6000 + p * 1000 + n, m_scale=0.0, noise=0.5)
    case.g[:, : min(n, 40)] = 0
    case.snapshot()
    ref = oracle_step(case, HP, step, p=p)
    q, nbytes = hip_update_pack(case, HP, step, C)
    if C == 1:
        got_fields = q[:, : nbytes].cpu().numpy()[:, : (n + 7) // 8]
    else:
        got_fields = q[:, : nbytes].cpu().numpy()
    assert np.array_equal(got_fields, ref["fields"]), "p-bit fields"
    assert untouched(q, nbytes)
    assert_close(case.m.cpu().numpy(), ref["m"], "momentum")
    nw = nwords(n)
    fb = (n * C + 7) // 8
    sum_out = guarded(1, nw * 8 if C == 1 else fb, case.device)
    pos, nz = guarded(1, nw * 8, case.device), guarded(1, nw * 8, case.device)
    lc.lc_pbit_sum_sign(q, q.stride(0), C, W, n, p, sum_out, pos, nz, step, lc.LC_TIE_ZERO)
    torch.cuda.synchronize()
    assert np.array_equal(sum_out[0, :fb].cpu().numpy(), ref["sum_fields"]), "field sums"
    assert untouched(sum_out, nw * 8 if C == 1 else fb)
    assert np.array_equal(words_of(pos, nw)[0], ref["pos"]) and np.array_equal(words_of(nz, nw)[0], ref["nz"])
    sum2 = guarded(1, nw * 8 if C == 1 else fb, case.device)
    lc.lc_pbit_sum_apply(q, q.stride(0), C, W, n, p, sum2, step, lc.LC_TIE_ZERO, case.theta, HP["lr"], HP["wd"],
                         None, 0, None, 0, lc.LC_F32, 0, HP["beta2"])
    torch.cuda.synchronize()
    assert np.array_equal(sum2[0, :fb].cpu().numpy(), ref["sum_fields"])
    assert_close(case.theta.cpu().numpy(), ref["theta"], "theta")


@pytest.mark.parametrize("p,W", [(2, 3), (4, 8), (4, 15), (7, 64), (8, 200)])
@pytest.mark.parametrize("n", [5, 4096 + 3, 16384 * 2 + 100])
def test_pbit_sum_from_1bit_rows(p, W, n):
    """The counts K as p-bit fields computed from 1-bit buffers (the form of the
    reduction-only workload), fused with apply and a one-stream momentum update."""
    C = lc.lc_container_bits(p)
    case = Case(n, W, seed=7000 + p + n, m_scale=0.0)
    ref = oracle_step(case, HP, 2, tie=orc.TIE_ALT, p=p)
    q, nbytes = hip_update_pack(case, HP, 2, 1, update_m=False)
    fb = (n * C + 7) // 8
    nw = nwords(n)
    s1, s2 = guarded(1, fb, case.device), guarded(1, fb, case.device)
    pos, nz = guarded(1, nw * 8, case.device), guarded(1, nw * 8, case.device)
    lc.lc_pbit_sum_sign(q, q.stride(0), 1, W, n, p, s1, pos, nz, 2, lc.LC_TIE_ALT)
    lc.lc_pbit_sum_apply(q, q.stride(0), 1, W, n, p, s2, 2, lc.LC_TIE_ALT, case.theta, HP["lr"], HP["wd"],
                         case.m, case.m.stride(0), case.g, case.g.stride(0), lc.LC_F32, 1, HP["beta2"])
    torch.cuda.synchronize()
    for s in (s1, s2):
        assert np.array_equal(s[0, :fb].cpu().numpy(), ref["sum_fields"]), "counts from 1-bit rows"
        assert untouched(s, fb)
    assert np.array_equal(words_of(pos, nw)[0], ref["pos"]) and np.array_equal(words_of(nz, nw)[0], ref["nz"])
    assert (words_of(nz, nw)[0][:-1] == np.uint64(2 ** 64 - 1)).all()         # TIE_ALT leaves no zero
    assert_close(case.theta.cpu().numpy(), ref["theta"], "theta")
    m = case.m.cpu().numpy()
    assert_close(m[0], ref["m"][0], "momentum of stream 0")
    assert np.array_equal(m[1:], case.m0[1:])                                  # n_m = 1: others untouched


@pytest.mark.parametrize("g_dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n_m", [1, 3])
@pytest.mark.parametrize("n", [777, 16384 + 4099])
def test_apply_with_momentum_streams(g_dtype, n_m, n):
    """lc_apply_update / lc_vote_apply_1bit with the momentum update done in the apply pass."""
    W = 4
    case = Case(n, W, seed=8000 + n, g_dtype=g_dtype, m_scale=0.0)
    ref = oracle_step(case, HP, 1)
    q, _ = hip_update_pack(case, HP, 1, 1, update_m=False)
    theta_a = case.theta.clone()
    m_a = clone_rows(case.m)
    lc.lc_vote_apply_1bit(q, q.stride(0) // 8, W, n, 1, lc.LC_TIE_ZERO, case.theta, HP["lr"], HP["wd"], case.m,
                          case.m.stride(0), case.g, case.g.stride(0), case.gd, n_m, HP["beta2"])
    nw = nwords(n)
    pos, nz = guarded(1, nw * 8, case.device), guarded(1, nw * 8, case.device)
    lc.lc_vote_1bit(q, q.stride(0) // 8, W, n, pos, nz, 1, lc.LC_TIE_ZERO)
    lc.lc_apply_update(theta_a, pos, nz, n, HP["lr"], HP["wd"], m_a, m_a.stride(0), case.g, case.g.stride(0), case.gd,
                       n_m, HP["beta2"])
    torch.cuda.synchronize()
    for th, mm in ((case.theta, case.m), (theta_a, m_a)):
        assert_close(th.cpu().numpy(), ref["theta"], "theta")
        got = mm.cpu().numpy()
        assert_close(got[:n_m], ref["m"][:n_m], "momentum")
        assert np.array_equal(got[n_m:], case.m0[n_m:])
    assert torch.equal(theta_a, case.theta) and torch.equal(m_a, case.m)      # fused == unfused, bit for bit


def test_apply_one_plane():
    """vote_nz = NULL: every element moves, -1 where the pos bit is clear."""
    n, W = 5000, 4
    case = Case(n, W, seed=8500, m_scale=0.0)
    ref = oracle_step(case, HP, 1, tie=orc.TIE_ALT)
    q, _ = hip_update_pack(case, HP, 1, 1, update_m=False)
    nw = nwords(n)
    pos = guarded(1, nw * 8, case.device)
    lc.lc_vote_1bit(q, q.stride(0) // 8, W, n, pos, None, 1, lc.LC_TIE_ALT)
    lc.lc_apply_update(case.theta, pos, None, n, HP["lr"], HP["wd"], None, 0, None, 0, lc.LC_F32, 0, HP["beta2"])
    torch.cuda.synchronize()
    assert_close(case.theta.cpu().numpy(), ref["theta"], "theta")


@pytest.mark.parametrize("W", [2, 3, 8, 16, 33])
@pytest.mark.parametrize("n", [1, 3, 4, 1023, 1024, 1025, 70001])
def test_momentum_avg(W, n):
    case = Case(n, W, seed=9000 + W + n, m_spread=1.0)
    ref = orc.momentum_avg(case.m0)
    lc.lc_momentum_avg(case.m, case.m.stride(0), W, n)
    torch.cuda.synchronize()
    got = case.m.cpu().numpy()
    for w in range(W):
        assert_close(got[w], ref, "averaged momentum row %d" % w)
    assert (got == got[0]).all()


def test_empty_range_is_a_noop():
    case = Case(64, 2, seed=1)
    q = guarded(2, 8, case.device)
    lc.lc_local_update_pack(case.g, case.g.stride(0), case.gd, case.m, case.m.stride(0), 2, 0, 0.9, 1, 0.99, 1, q,
                            q.stride(0), 1, lc.LC_ZERO_ALT)
    lc.lc_vote_apply_1bit(q, q.stride(0) // 8, 2, 0, 1, lc.LC_TIE_ZERO, case.theta, 1e-4, 0.1, None, 0, None, 0,
                          lc.LC_F32, 0, 0.99)
    lc.lc_momentum_avg(case.m, case.m.stride(0), 2, 0)
    torch.cuda.synchronize()
    assert (q == SENTINEL).all().item()
    assert np.array_equal(case.m.cpu().numpy(), case.m0) and np.array_equal(case.theta.cpu().numpy(), case.theta0)


def test_multi_step_trajectory():
    """Four consecutive steps (odd and even iterations) with state carried on the GPU;
    the oracle restarts each step from the GPU's fp32 state, so errors cannot hide in drift."""
    n, W = 50000, 4
    case = Case(n, W, seed=10000)
    for step in range(1, 5):
        case.g.copy_(torch.randn(W, n, generator=torch.Generator(device="cuda").manual_seed(step), device="cuda") * 1e-3)
        case.snapshot()
        out = run_1bit(case, step)
        check_1bit(out, oracle_step(case, HP, step))


def test_side_stream_and_read_only_inputs():
    """Calls on a non-default stream, given as the `stream` argument, while the default
    stream is busy; g and q are read-only for the calls that take them as inputs."""
    n, W = 300000 + 13, 8
    case = Case(n, W, seed=11000, m_spread=1.0)
    ref = oracle_step(case, HP, 3)
    side = torch.cuda.Stream()
    nw = nwords(n)
    q = guarded(W, nw * 8, case.device)
    g_before = case.g.clone()
    busy = torch.randn(1 << 24, device="cuda")
    side.wait_stream(torch.cuda.current_stream())
    for _ in range(20):
        busy = busy * 1.0001 + 1.0                           # keeps the default stream occupied
    lc.lc_local_update_pack(case.g, case.g.stride(0), case.gd, case.m, case.m.stride(0), W, n, HP["beta1"], 1,
                            HP["beta2"], 1, q, q.stride(0), 3, lc.LC_ZERO_ALT, stream=side)
    q_before = None
    with torch.cuda.stream(side):
        q_before = q.clone()
    lc.lc_vote_apply_1bit(q, q.stride(0) // 8, W, n, 3, lc.LC_TIE_ZERO, case.theta, HP["lr"], HP["wd"], None, 0, None, 0,
                          lc.LC_F32, 0, HP["beta2"], stream=side.cuda_stream)
    side.synchronize()
    torch.cuda.synchronize()
    assert np.array_equal(words_of(q, nw), ref["words"])
    assert_close(case.theta.cpu().numpy(), ref["theta"], "theta")
    assert_close(case.m.cpu().numpy(), ref["m"], "momentum")
    assert torch.equal(case.g, g_before) and torch.equal(q, q_before)


def test_per_tensor_calls_equal_one_arena_call():
    """A model as one flat arena, or one call per tensor at 64-aligned offsets (per-group
    learning rates need that): the same bits either way."""
    sizes = [64 * 37, 768, 768 * 5, 64, 2304, 64 * 129, 768 * 3 + 64 * 2, 4096 * 3, 1024 + 64]
    n, W = sum(sizes), 4
    a = Case(n, W, seed=12000, m_scale=0.0)
    b = Case(n, W, seed=12000, m_scale=0.0)
    nw = n // 64
    qa, qb = guarded(W, nw * 8, a.device), guarded(W, nw * 8, b.device)
    lc.lc_local_update_pack(a.g, a.g.stride(0), a.gd, a.m, a.m.stride(0), W, n, HP["beta1"], 1, HP["beta2"], 1, qa,
                            qa.stride(0), 1, lc.LC_ZERO_ALT)
    lc.lc_vote_apply_1bit(qa, qa.stride(0) // 8, W, n, 1, lc.LC_TIE_ZERO, a.theta, HP["lr"], HP["wd"], None, 0, None, 0,
                          lc.LC_F32, 0, HP["beta2"])
    off = 0
    for sz in sizes:
        lc.lc_local_update_pack(b.g[:, off:], b.g.stride(0), b.gd, b.m[:, off:], b.m.stride(0), W, sz, HP["beta1"], 1,
                                HP["beta2"], 1, qb[:, off // 8:], qb.stride(0), 1, lc.LC_ZERO_ALT)
        lc.lc_vote_apply_1bit(qb[:, off // 8:], qb.stride(0) // 8, W, sz, 1, lc.LC_TIE_ZERO, b.theta[off:], HP["lr"],
                              HP["wd"], None, 0, None, 0, lc.LC_F32, 0, HP["beta2"])
        off += sz
    torch.cuda.synchronize()
    assert torch.equal(qa, qb) and torch.equal(a.theta, b.theta) and torch.equal(a.m, b.m)
    check = oracle_step(a, HP, 1)
    assert np.array_equal(words_of(qa, nw), check["words"])
    assert_close(a.theta.cpu().numpy(), check["theta"], "theta")


def test_errors_leave_buffers_untouched():
    """Argument errors are found on the host before any launch: nothing is written."""
    n, W = 5000, 4
    case = Case(n, W, seed=13000)
    q = guarded(W, nwords(n) * 8, case.device)
    calls = [
        lambda: lc.lc_local_update_pack(case.g, case.g.stride(0), case.gd, case.m[:, 1:], case.m.stride(0), W, n - 1, 0.9,
                                        1, 0.99, 1, q, q.stride(0), 1, lc.LC_ZERO_ALT, check=False),       # m misaligned
        lambda: lc.lc_local_update_pack(case.g, case.g.stride(0), case.gd, case.m, case.m.stride(0), W, n, 0.9, 1, 0.99,
                                        3, q, q.stride(0), 1, lc.LC_ZERO_ALT, check=False),                # bad width
        lambda: lc.lc_pbit_sum_apply(q, q.stride(0), 1, 16, n, 4, None, 1, lc.LC_TIE_ZERO, case.theta, 1e-4, 0.1, None,
                                     0, None, 0, lc.LC_F32, 0, 0.99, check=False),                         # 16 workers, p = 4
        lambda: lc.lc_vote_apply_1bit(q, q.stride(0) // 8, W, n, 1, lc.LC_TIE_ZERO, case.theta[1:], 1e-4, 0.1, None, 0,
                                      None, 0, lc.LC_F32, 0, 0.99, check=False),                           # theta misaligned
        lambda: lc.lc_momentum_avg(case.m[:, 2:], case.m.stride(0), W, n - 2, check=False),                # 8-byte aligned only
    ]
    want = [lc.LC_ERR_ALIGN, lc.LC_ERR_MODE, lc.LC_ERR_RANGE, lc.LC_ERR_ALIGN, lc.LC_ERR_ALIGN]
    assert [c() for c in calls] == want
    torch.cuda.synchronize()
    assert (q == SENTINEL).all().item()
    assert np.array_equal(case.m.cpu().numpy(), case.m0) and np.array_equal(case.theta.cpu().numpy(), case.theta0)


@pytest.mark.parametrize("W", [2, 3, 8, 16])
@pytest.mark.parametrize("n", [1, 5, 1023, 1024, 1025, 200003])
def test_momentum_divergence(W, n):
    """Section 5.1's metric: max over elements of the std across workers, fp64."""
    case = Case(n, W, seed=14000 + W + n, m_spread=0.3)
    out = torch.full((1,), -1.0, dtype=torch.float64, device="cuda")
    lc.lc_momentum_divergence(case.m, case.m.stride(0), W, n, out)
    torch.cuda.synchronize()
    ref = orc.momentum_divergence(case.m0)
    assert ref > 0 and abs(float(out[0]) - ref) <= 1e-12 * ref
    lc.lc_momentum_avg(case.m, case.m.stride(0), W, n)
    lc.lc_momentum_divergence(case.m, case.m.stride(0), W, n, out)
    torch.cuda.synchronize()
    assert float(out[0]) == 0.0                                              # synchronised: no divergence left
    lc.lc_momentum_divergence(case.m, case.m.stride(0), W, 0, out)
    torch.cuda.synchronize()
    assert float(out[0]) == 0.0


@pytest.mark.parametrize("W", [3, 16, 40, 70])
def test_momentum_divergence_special_values(W):
    """Elements that hold a NaN or an infinity have no standard deviation and take no part in the
    maximum (the comparison with a NaN is false on both sides); denormals and huge values do."""
    n = 5000
    case = Case(n, W, seed=14300 + W, m_spread=0.3)
    case.m[0, 10] = float("nan")
    case.m[W - 1, 11] = float("inf")
    case.m[1, 12] = -float("inf")
    case.m[:, 300] = torch.linspace(-1e-41, 1e-41, W)          # denormals
    case.m[:, 4000] = torch.linspace(-1.0, 1.0, W) * 1e18       # the maximum sits here
    case.m[:, 256 * 19 + 3] = float("nan")                       # a whole column, in the ragged last tile
    case.snapshot()
    out = torch.full((1,), -1.0, dtype=torch.float64, device="cuda")
    lc.lc_momentum_divergence(case.m, case.m.stride(0), W, n, out)
    torch.cuda.synchronize()
    ref = orc.momentum_divergence(case.m0)
    assert ref > 1e17 and np.isfinite(ref) and abs(float(out[0]) - ref) <= 1e-12 * ref
    end_t = torch.tensor([4, 63, (n + 63) // 64], dtype=torch.int32, device="cuda")
    outg = torch.full((3,), -1.0, dtype=torch.float64, device="cuda")
    lc.lc_momentum_divergence_groups(case.m, case.m.stride(0), W, n, end_t, 3, outg)
    torch.cuda.synchronize()
    for s, (lo, hi) in enumerate(((0, 256), (256, 4032), (4032, n))):
        r = orc.momentum_divergence(case.m0[:, lo:hi])
        assert abs(float(outg[s]) - r) <= 1e-12 * r, (s, float(outg[s]), r)


@pytest.mark.parametrize("W", [2, 5, 16])
def test_momentum_divergence_per_group(W):
    """The same metric for every segment of a group table in one launch (Figure 6 is per
    layer): each value against the oracle run on that segment alone.  Segments of 64
    elements, boundaries inside a wave's 256 elements, empty segments, a ragged end; the
    spread differs per segment so that a value landing in the wrong slot shows."""
    ends64 = [1, 2, 2, 7, 40, 41, 41, 300, 1000, 1003]
    n = 64 * 1003 - 29
    case = Case(n, W, seed=14500 + W, m_spread=0.3)
    G = len(ends64)
    bounds = [0] + [min(e * 64, n) for e in ends64]
    for s in range(G):
        case.m[:, bounds[s]:bounds[s + 1]] *= 2.0 ** (s % 5)
    case.snapshot()
    end_t = torch.tensor(ends64, dtype=torch.int32, device="cuda")
    out = torch.full((G,), -1.0, dtype=torch.float64, device="cuda")
    lc.lc_momentum_divergence_groups(case.m, case.m.stride(0), W, n, end_t, G, out)
    whole = torch.full((1,), -1.0, dtype=torch.float64, device="cuda")
    lc.lc_momentum_divergence(case.m, case.m.stride(0), W, n, whole)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    for s in range(G):
        lo, hi = bounds[s], bounds[s + 1]
        ref = orc.momentum_divergence(case.m0[:, lo:hi]) if hi > lo else 0.0
        assert abs(got[s] - ref) <= 1e-12 * ref, "segment %d [%d, %d): %r vs %r" % (s, lo, hi, got[s], ref)
    assert got.max() == float(whole[0]) and len(set(got.tolist())) >= 7
    assert lc.lc_momentum_divergence_groups(case.m, case.m.stride(0), W, n, None, G, out, check=False) == lc.LC_ERR_NULL
    assert lc.lc_momentum_divergence_groups(case.m, case.m.stride(0), W, n, end_t, 0, out, check=False) == lc.LC_ERR_SIZE


@pytest.mark.parametrize("G,W,longest", [(64, 3, 6), (65, 8, 6), (200, 16, 6), (1024, 4, 6), (1025, 5, 6), (3000, 2, 6),
                                         (700, 33, 6), (300, 70, 6), (200, 16, 400), (40, 4, 9000)])
def test_momentum_divergence_many_groups(G, W, longest):
    """Group tables on either side of what the kernel resolves with lane masks (up to 1024
    groups) and of what it bisects, with every row count class (rows held in registers up
    to 64, read twice beyond): random segment lengths of 0 to `longest` blocks -- short ones,
    so that most waves straddle a boundary, and long ones, so that the launch has several
    thousand workgroups -- a ragged end, each value against the oracle on its own segment."""
    rng = np.random.default_rng(G * 7 + W)
    ends64 = np.cumsum(rng.integers(0, longest + 1, G)).astype(np.int64)
    n = int(ends64[-1]) * 64 - 37
    case = Case(n, W, seed=14700 + G + W, m_spread=0.3)
    bounds = [0] + [min(int(e) * 64, n) for e in ends64]
    scale = torch.ones(n, device="cuda")
    for s in range(G):
        scale[bounds[s]:bounds[s + 1]] = 2.0 ** (s % 7)
    case.m *= scale
    case.snapshot()
    end_t = torch.tensor(ends64, dtype=torch.int64).to(torch.int32).cuda()
    out = torch.full((G,), -1.0, dtype=torch.float64, device="cuda")
    lc.lc_momentum_divergence_groups(case.m, case.m.stride(0), W, n, end_t, G, out)
    whole = torch.full((1,), -1.0, dtype=torch.float64, device="cuda")
    lc.lc_momentum_divergence(case.m, case.m.stride(0), W, n, whole)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    for s in range(G):
        lo, hi = bounds[s], bounds[s + 1]
        ref = orc.momentum_divergence(case.m0[:, lo:hi]) if hi > lo else 0.0
        assert abs(got[s] - ref) <= 1e-12 * ref, "segment %d of %d [%d, %d): %r vs %r" % (s, G, lo, hi, got[s], ref)
    assert got.max() == float(whole[0])
    ref = orc.momentum_divergence(case.m0)
    assert abs(float(whole[0]) - ref) <= 1e-12 * ref


def test_momentum_sync_ranges_policy():
    """Selected ranges only, and only on every k-th iteration (Section 6.2: head and
    embedding every ten iterations)."""
    n, W = 64 * 300, 4
    case = Case(n, W, seed=15000, m_spread=1.0)
    offsets, sizes = [0, 64 * 100, 64 * 250], [64 * 10, 64 * 7 + 12, 64 * 50]
    for step in (1, 7, 9):
        lc.lc_momentum_sync_ranges(case.m, case.m.stride(0), W, offsets, sizes, 3, step, 10)
    torch.cuda.synchronize()
    assert np.array_equal(case.m.cpu().numpy(), case.m0)                     # not a synchronisation step
    lc.lc_momentum_sync_ranges(case.m, case.m.stride(0), W, offsets, sizes, 3, 20, 10)
    torch.cuda.synchronize()
    got = case.m.cpu().numpy()
    inside = np.zeros(n, bool)
    for o, sz in zip(offsets, sizes):
        inside[o:o + sz] = True
        ref = orc.momentum_avg(case.m0[:, o:o + sz])
        for w in range(W):
            assert_close(got[w, o:o + sz], ref, "averaged range")
    assert np.array_equal(got[:, ~inside], case.m0[:, ~inside])              # everything else untouched


@pytest.mark.parametrize("W,n_ranges", [(2, 5), (4, 32), (8, 33), (16, 100), (3, 70)])
def test_momentum_sync_many_ranges(W, n_ranges):
    """Selective synchronisation over more ranges than one launch carries: ranges of 0 to
    3000 elements (lengths that are no multiple of 4, empty ones, one longer than a few
    tiles) with gaps between them.  Every range equals lc_momentum_avg on that range bit for
    bit and the oracle within tolerance; the gaps keep their values."""
    rng = np.random.default_rng(15100 + W + n_ranges)
    offsets, sizes, at = [], [], 0
    for r in range(n_ranges):
        at += 4 * int(rng.integers(0, 40))
        sz = int(rng.choice([0, 1, 3, 4, 255, 256, 257, 1000, 3000, 70001])) if r % 7 else int(rng.integers(0, 3000))
        offsets.append(at)
        sizes.append(sz)
        at += (sz + 3) // 4 * 4
    n = at + 64
    case = Case(n, W, seed=15200 + W, m_spread=1.0)
    twin = clone_rows(case.m)
    lc.lc_momentum_sync_ranges(case.m, case.m.stride(0), W, offsets, sizes, n_ranges, 30, 10)
    for o, sz in zip(offsets, sizes):
        if sz:
            lc.lc_momentum_avg(twin[:, o:], twin.stride(0), W, sz)
    torch.cuda.synchronize()
    got = case.m.cpu().numpy()
    assert np.array_equal(got, twin.cpu().numpy())                           # one launch per batch == one launch per range
    inside = np.zeros(n, bool)
    for o, sz in zip(offsets, sizes):
        inside[o:o + sz] = True
        if sz:
            ref = orc.momentum_avg(case.m0[:, o:o + sz])
            for w in range(W):
                assert_close(got[w, o:o + sz], ref, "averaged range")
    assert np.array_equal(got[:, ~inside], case.m0[:, ~inside])
    assert inside.sum() > 0 and (~inside).sum() > 0


def test_hip_graph_replay_matches_eager():
    """The library only launches kernels (no memsets, no allocation, no synchronisation),
    so a step can be captured into a HIP graph.  Several replays, with eager work and
    synchronisations in between, must each equal the eager result bit for bit."""
    n, W = 200000 + 77, 4
    eager = Case(n, W, seed=16000, m_spread=1.0)
    graph = Case(n, W, seed=16000, m_spread=1.0)
    nw = nwords(n)
    mean = torch.zeros(W, dtype=torch.float64, device="cuda")
    ws = torch.zeros(W * lc.LC_L1_WORKSPACE_WORDS, dtype=torch.int64, device="cuda")
    lv = torch.zeros((W, (n + 127) // 64 * 64), dtype=torch.uint8, device="cuda")

    def step(case, q, stream):
        lc.lc_local_update_pack(case.g, case.g.stride(0), case.gd, case.m, case.m.stride(0), W, n, HP["beta1"], 1,
                                HP["beta2"], 1, q, q.stride(0), 1, lc.LC_ZERO_ALT, stream=stream)
        lc.lc_vote_apply_1bit(q, q.stride(0) // 8, W, n, 1, lc.LC_TIE_ZERO, case.theta, HP["lr"], HP["wd"], None, 0, None,
                              0, lc.LC_F32, 0, HP["beta2"], stream=stream)
        lc.lc_l1_mean_abs(case.g, case.g.stride(0), case.gd, case.m, case.m.stride(0), W, n, HP["beta1"], mean, ws,
                          stream=stream)                      # zeroes its workspace with a kernel, not a memset
        lc.lc_l1_quantize_pack(case.g, case.g.stride(0), case.gd, case.m, case.m.stride(0), W, n, HP["beta1"], 0,
                               HP["beta2"], 15, mean, lv, lv.stride(0), stream=stream)
        lc.lc_momentum_divergence(case.m, case.m.stride(0), W, n, div, stream=stream)   # clears its slot with a kernel too
        lc.lc_momentum_divergence_groups(case.m, case.m.stride(0), W, n, ends, 3, divg, stream=stream)
        lc.lc_momentum_sync_ranges(case.m, case.m.stride(0), W, [0, 4096, 70000], [1000, 30001, 64], 3, 10, 5, stream=stream)
        lc.lc_momentum_avg(case.m[:, 100000:], case.m.stride(0), W, n - 100000, stream=stream)

    div = torch.zeros(1, dtype=torch.float64, device="cuda")
    divg = torch.zeros(3, dtype=torch.float64, device="cuda")
    ends = torch.tensor([100, 2000, (n + 63) // 64], dtype=torch.int32, device="cuda")
    qe, qg = guarded(W, nw * 8, "cuda"), guarded(W, nw * 8, "cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(graph, qg, side)                                 # warm-up outside capture, then restore the state
        side.synchronize()
        graph.theta.copy_(torch.from_numpy(graph.theta0).cuda())
        graph.m.copy_(torch.from_numpy(graph.m0).cuda())
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            step(graph, qg, side)
    torch.cuda.synchronize()
    for replay in range(4):
        step(eager, qe, None)
        lv_eager = lv.clone()
        mean_eager = mean.clone()
        div_eager, divg_eager = div.clone(), divg.clone()
        torch.cuda.synchronize()
        lv.zero_()
        mean.zero_()
        div.fill_(-1.0)
        divg.fill_(-1.0)
        g.replay()
        torch.cuda.synchronize()
        assert div_eager.item() > 0 and torch.equal(div, div_eager) and torch.equal(divg, divg_eager), "replay %d: divergence" % replay
        assert torch.equal(qe, qg), "replay %d: packed words" % replay
        assert torch.equal(eager.theta, graph.theta) and torch.equal(eager.m, graph.m), "replay %d" % replay
        assert torch.equal(lv, lv_eager) and torch.equal(mean, mean_eager), "replay %d: L1 levels" % replay
        busy = torch.randn(1 << 20, device="cuda").sum().item()          # eager work between replays
        assert busy == busy


@pytest.mark.parametrize("ragged_tail", [0, 37])
def test_groups_in_one_launch_equal_per_tensor_calls(ragged_tail):
    """Per-group learning rate / weight decay: one launch with a device table of segments
    against one call per tensor, and both against the oracle."""
    sizes = [64 * 37, 768, 768 * 5, 64, 2304, 64 * 129, 768 * 3 + 64 * 2, 4096 * 3, 1024 + 64, 64 * 40 + ragged_tail]
    lrs = [1e-4, 3e-3, 1e-4, 3e-2, 1e-4, 2e-4, 3e-3, 1e-4, 5e-5, 3e-3]
    wds = [0.1, 0.0, 0.1, 0.01, 0.0, 0.1, 1.0, 0.1, 0.1, 0.0]
    n, W = sum(sizes), 4
    a = Case(n, W, seed=17000, m_scale=0.0)
    b = Case(n, W, seed=17000, m_scale=0.0)
    nw = nwords(n)
    q = guarded(W, nw * 8, a.device)
    lc.lc_local_update_pack(a.g, a.g.stride(0), a.gd, a.m, a.m.stride(0), W, n, HP["beta1"], 0, HP["beta2"], 1, q,
                            q.stride(0), 2, lc.LC_ZERO_ALT)
    ends, off = [], 0
    for sz in sizes:
        off += sz
        ends.append((off + 63) // 64)
    end64 = torch.tensor(ends, dtype=torch.int32, device="cuda")
    lr_t = torch.tensor(lrs, dtype=torch.float32, device="cuda")
    wd_t = torch.tensor(wds, dtype=torch.float32, device="cuda")
    lc.lc_vote_apply_1bit_groups(q, q.stride(0) // 8, W, n, 2, lc.LC_TIE_ZERO, a.theta, end64, lr_t, wd_t, len(sizes))
    off = 0
    ref = oracle_step(a, HP, 2)
    want = np.empty(n, np.float64)
    for sz, lr, wd in zip(sizes, lrs, wds):
        lc.lc_vote_apply_1bit(q[:, off // 8:], q.stride(0) // 8, W, sz, 2, lc.LC_TIE_ZERO, b.theta[off:], lr, wd, None, 0,
                              None, 0, lc.LC_F32, 0, HP["beta2"])
        want[off:off + sz] = orc.apply(a.theta0[off:off + sz], ref["u"][off:off + sz], lr, wd)
        off += sz
    torch.cuda.synchronize()
    assert torch.equal(a.theta, b.theta)
    assert_close(a.theta.cpu().numpy(), want, "theta with per-group rates")
    assert lc.lc_vote_apply_1bit_groups(q, q.stride(0) // 8, W, n, 2, lc.LC_TIE_ZERO, a.theta, None, lr_t, wd_t, 3,
                                        check=False) == lc.LC_ERR_NULL
    assert lc.lc_vote_apply_1bit_groups(q, q.stride(0) // 8, W, n, 2, lc.LC_TIE_ZERO, a.theta, end64, lr_t, wd_t, 0,
                                        check=False) == lc.LC_ERR_SIZE


@pytest.mark.parametrize("kind", ["p4_fields", "p3_from_bits", "ternary"])
def test_groups_for_field_sums_and_ternary_votes(kind):
    """The per-group table on the other aggregation inputs: p-bit fields, 1-bit rows summed
    as p-bit counts, and ternary planes -- one launch against the oracle applied segment by
    segment with each segment's rate and decay."""
    sizes = [64 * 5, 768, 64, 64 * 130, 2304, 64 * 3, 4096 * 2 + 64, 64 * 9 + 21]
    lrs = [1e-4, 3e-3, 3e-2, 1e-4, 2e-4, 5e-5, 1e-4, 3e-3]
    wds = [0.1, 0.0, 0.01, 0.1, 1.0, 0.1, 0.0, 0.1]
    n, W, G = sum(sizes), 4, len(sizes)
    case = Case(n, W, seed=17100, noise=2.0)
    case.g[:, ::7] = 0                                                   # exact zeros: ties and zero rule at work
    case.m[:, ::7] = 0
    case.snapshot()
    ends, off = [], 0
    for sz in sizes:
        off += sz
        ends.append((off + 63) // 64)
    end64 = torch.tensor(ends, dtype=torch.int32, device="cuda")
    lr_t = torch.tensor(lrs, dtype=torch.float32, device="cuda")
    wd_t = torch.tensor(wds, dtype=torch.float32, device="cuda")
    nw = nwords(n)
    step = 3
    if kind == "ternary":
        pos, nz = guarded(W, nw * 8, "cuda"), guarded(W, nw * 8, "cuda")
        lc.lc_local_update_pack_ternary(case.g, case.g.stride(0), case.gd, case.m, case.m.stride(0), W, n, HP["beta1"], 0,
                                        HP["beta2"], pos, nz, pos.stride(0) // 8)
        lc.lc_vote_apply_ternary_groups(pos, nz, pos.stride(0) // 8, W, n, case.theta, end64, lr_t, wd_t, G)
        u = orc.step_ternary(case.theta0, case.m0, case.g0, **HP)["u"]
    else:
        p, bits = (4, 4) if kind == "p4_fields" else (3, 1)
        nbytes = (n * bits + 7) // 8
        q = guarded(W, nbytes, "cuda")
        lc.lc_local_update_pack(case.g, case.g.stride(0), case.gd, case.m, case.m.stride(0), W, n, HP["beta1"], 0,
                                HP["beta2"], bits, q, q.stride(0), step, lc.LC_ZERO_ALT)
        C = lc.lc_container_bits(p)
        ksum = guarded(1, (n * C + 7) // 8, "cuda")
        lc.lc_pbit_sum_apply_groups(q, q.stride(0), bits, W, n, p, ksum, step, lc.LC_TIE_ZERO, case.theta, end64, lr_t,
                                    wd_t, G)
        ref = orc.step_pbit(case.theta0, case.m0, case.g0, p=p, step=step, **HP)
        u = ref["u"]
        assert np.array_equal(ksum[0, :(n * C + 7) // 8].cpu().numpy(), ref["sum_fields"])
    torch.cuda.synchronize()
    want, off = np.empty(n, np.float64), 0
    for sz, lr, wd in zip(sizes, lrs, wds):
        want[off:off + sz] = orc.apply(case.theta0[off:off + sz], u[off:off + sz], lr, wd)
        off += sz
    assert (u == 0).any() and (u == 1).any() and (u == -1).any()
    assert_close(case.theta.cpu().numpy(), want, "theta with per-group rates (%s)" % kind)


@pytest.mark.parametrize("p,W,n", [(2, 3, 4099), (4, 8, 70001), (4, 15, 255), (7, 100, 33333), (8, 255, 5000), (3, 6, 1)])
@pytest.mark.parametrize("n_m", [0, 2])
def test_count_apply_after_a_summing_allreduce(p, W, n, n_m):
    """The direct-allreduce route of Section 3: the collective delivers the summed fields K,
    the library compares them with the worker count and applies.  The sums come from the
    oracle (what a summing allreduce over the W field buffers yields)."""
    step, tie = 5, lc.LC_TIE_ZERO if n % 2 else lc.LC_TIE_ALT
    case = Case(n, W, seed=18000 + p + W, noise=3.0)
    case.g[:, ::5] = 0
    case.m[:, ::5] = 0
    case.snapshot()
    ref = orc.step_pbit(case.theta0, case.m0, case.g0, p=p, step=step, tie=tie, **HP)
    C = lc.lc_container_bits(p)
    k = guarded(1, (n * C + 7) // 8, "cuda")
    k[0, :(n * C + 7) // 8] = torch.from_numpy(ref["sum_fields"]).cuda()
    n_rows = min(n_m, W)
    lc.lc_count_apply(k, C, n, W, step, tie, case.theta, HP["lr"], HP["wd"], case.m if n_rows else None, case.m.stride(0),
                      case.g if n_rows else None, case.g.stride(0), case.gd, n_rows, HP["beta2"])
    torch.cuda.synchronize()
    assert_close(case.theta.cpu().numpy(), ref["theta"], "theta from summed fields")
    assert_close(case.m[:n_rows].cpu().numpy(), ref["m"][:n_rows], "momentum rows")
    assert np.array_equal(case.m[n_rows:].cpu().numpy(), case.m0[n_rows:])
    assert untouched(k, (n * C + 7) // 8)
    assert lc.lc_count_apply(k, C, n, 1 << C, step, tie, case.theta, 1e-4, 0.1, None, 0, None, 0, lc.LC_F32, 0, 0.99,
                             check=False) == lc.LC_ERR_RANGE
    assert lc.lc_count_apply(k, 1, n, 1, step, tie, case.theta, 1e-4, 0.1, None, 0, None, 0, lc.LC_F32, 0, 0.99,
                             check=False) == lc.LC_ERR_MODE


def test_count_apply_on_summed_l1_levels():
    """The 8-bit allreduce of Appendix F.1 sums level bytes; total = 2 W L."""
    n, W, L, step = 50021, 8, 15, 4
    case = Case(n, W, seed=18100, m_spread=1.0)
    ref = orc.step_l1(case.theta0, case.m0, case.g0, L=L, step=step, tie=orc.TIE_ALT, **HP)
    k = guarded(1, n, "cuda")
    k[0, :n] = torch.from_numpy(ref["K"].astype(np.uint8)).cuda()
    lc.lc_count_apply(k, 8, n, 2 * W * L, step, lc.LC_TIE_ALT, case.theta, HP["lr"], HP["wd"], None, 0, None, 0, lc.LC_F32, 0,
                      HP["beta2"])
    torch.cuda.synchronize()
    assert (ref["S"] == 0).any()
    assert_close(case.theta.cpu().numpy(), ref["theta"], "theta from summed level bytes")


def test_momentum_divergence_per_group_degenerate_cases():
    """One worker has no divergence; n = 0 writes zeros; a single group equals the plain call."""
    case = Case(5000, 1, seed=14600)
    end_t = torch.tensor([10, 79], dtype=torch.int32, device="cuda")
    out = torch.full((2,), -1.0, dtype=torch.float64, device="cuda")
    lc.lc_momentum_divergence_groups(case.m, case.m.stride(0), 1, 5000, end_t, 2, out)
    torch.cuda.synchronize()
    assert out.tolist() == [0.0, 0.0]
    many = Case(70001, 6, seed=14601, m_spread=0.4)
    out.fill_(-1.0)
    lc.lc_momentum_divergence_groups(many.m, many.m.stride(0), 6, 0, end_t, 2, out)
    torch.cuda.synchronize()
    assert out.tolist() == [0.0, 0.0]
    one_end = torch.tensor([(70001 + 63) // 64], dtype=torch.int32, device="cuda")
    a = torch.zeros(1, dtype=torch.float64, device="cuda")
    b = torch.zeros(1, dtype=torch.float64, device="cuda")
    lc.lc_momentum_divergence_groups(many.m, many.m.stride(0), 6, 70001, one_end, 1, a)
    lc.lc_momentum_divergence(many.m, many.m.stride(0), 6, 70001, b)
    torch.cuda.synchronize()
    assert a.item() == b.item() and a.item() > 0
