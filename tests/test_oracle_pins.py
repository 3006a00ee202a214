"""Pins for the CPU oracle: every function of oracle/ is checked against something
other than itself -- the hand-enumerated case, values the paper prints, exact rational
arithmetic on tiny inputs, closed forms, invariants and brute force.  No GPU needed."""
import itertools
import math
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle as orc
from conftest import read_golden


def _ints(s):
    return [int(x) for x in s.split()]


def _hex(s):
    return [int(x, 16) for x in s.split()]


SIGN = {"+": 1.0, "-": -1.0, "0": 0.0}


# --------------------------------------------------------------------------------------
# hand-enumerated case (tests/golden/hand_case_w3_w4_n8.txt)
# --------------------------------------------------------------------------------------
@pytest.fixture(scope="module")
def hand():
    gold = read_golden("hand_case_w3_w4_n8.txt")
    g = np.array([[SIGN[c] for c in gold["g%d" % w].split()] for w in range(4)], np.float32)
    return gold, g


@pytest.mark.parametrize("step", [1, 2])
@pytest.mark.parametrize("beta1", [0.9, 0.5, 0.0])
def test_hand_case_words(hand, step, beta1):
    gold, g = hand
    m = np.zeros(8, np.float32)
    for w in range(4):
        s = orc.local_sign(m, g[w], beta1)
        assert s.tolist() == [int(x) for x in g[w]]
        words = orc.pack_1bit(orc.zero_rule(s, step))
        assert words.tolist() == [int(gold["step%d.word%d" % (step, w)], 16)]


@pytest.mark.parametrize("step", [1, 2])
@pytest.mark.parametrize("W", [3, 4])
def test_hand_case_vote(hand, step, W):
    gold, g = hand
    theta = np.zeros(8, np.float32)
    m = np.zeros((W, 8), np.float32)
    hp = dict(beta1=0.9, beta2=0.99, lr=1e-4, wd=0.0, step=step)
    r = orc.step_1bit(theta, m, g[:W], tie=orc.TIE_ZERO, **hp)
    key = "step%d.W%d." % (step, W)
    assert r["K"].tolist() == _ints(gold[key + "K"])
    assert r["S"].tolist() == _ints(gold[key + "S"])
    if W == 3:
        assert [int(r["pos"][0]), int(r["nz"][0])] == [int(gold[key + "pos"], 16),
                                                       int(gold[key + "nz"], 16)]
    else:
        assert int(r["pos"][0]) == int(gold[key + "tie_zero.pos"], 16)
        assert int(r["nz"][0]) == int(gold[key + "tie_zero.nz"], 16)
        r = orc.step_1bit(theta, m, g[:W], tie=orc.TIE_ALT, **hp)
        assert int(r["pos"][0]) == int(gold[key + "tie_alt.pos"], 16)
        assert int(r["nz"][0]) == int(gold[key + "tie_alt.nz"], 16)
    # with wd = 0 and theta = 0 the new parameter is exactly -lr * u
    assert np.array_equal(r["theta"], np.float64(np.float32(1e-4)) * -r["u"])


def test_hand_case_p4_fields(hand):
    gold, g = hand
    theta = np.zeros(8, np.float32)
    m = np.zeros((3, 8), np.float32)
    r = orc.step_pbit(theta, m, g[:3], p=4, beta1=0.9, beta2=0.99, lr=1e-4, wd=0.0, step=1)
    for w in range(3):
        assert r["fields"][w].tolist() == _hex(gold["step1.p4.fields%d" % w])
    assert r["sum_fields"].tolist() == _hex(gold["step1.p4.W3.sum"])
    assert r["K"].tolist() == _ints(gold["step1.W3.K"])


# --------------------------------------------------------------------------------------
# values the paper prints
# --------------------------------------------------------------------------------------
def test_bit_budget_from_paper():
    gold = read_golden("paper_printed_values.txt")
    b = np.ones((1, 1), np.uint8)
    for W in (8, 64):
        p = int(gold["bits_for_workers.%d" % W])
        assert p == int(math.log2(W)) + 1
        bits = np.ones((W, 3), np.uint8)
        K, S, u = orc.count_sign(bits, 1, p=p)          # accepted, and K reaches W
        assert K.tolist() == [W] * 3 and S.tolist() == [W] * 3 and u.tolist() == [1] * 3
        with pytest.raises(orc.OracleError):
            orc.count_sign(bits, 1, p=p - 1)            # one bit fewer cannot hold W
    ok, bad = int(gold["p4.max_workers_ok"]), int(gold["p4.first_workers_rejected"])
    orc.count_sign(np.repeat(b, ok, 0), 1, p=4)
    with pytest.raises(orc.OracleError) as e:
        orc.count_sign(np.repeat(b, bad, 0), 1, p=4)
    assert e.value.code == orc.ERR_RANGE
    orc.count_sign(np.repeat(b, int(gold["p8.workers_ok"]), 0), 1, p=8)
    for p in (-1, 9):                                   # no such field width, however few the workers
        with pytest.raises(orc.OracleError) as e:
            orc.count_sign(b, 1, p=p)
        assert e.value.code == orc.ERR_RANGE
    with pytest.raises(orc.OracleError) as e:           # a vote needs a voter
        orc.count_sign(np.ones((0, 3), np.uint8), 1)
    assert e.value.code == orc.ERR_ARG
    for call in (lambda: orc.level_sum_sign(np.zeros((0, 3), np.uint8), 15, 1),
                 lambda: orc.level_sum_sign(np.zeros((2, 3), np.uint8), 0, 1),
                 lambda: orc.ternary_vote(np.zeros((0, 3), np.int8))):
        with pytest.raises(orc.OracleError) as e:
            call()
        assert e.value.code == orc.ERR_ARG


def test_whole_step_range_rules():
    """The p-bit step serves at most 2^p - 1 workers with p from 1 to 8 (Section 3's count of
    bits); the level step needs the summed bytes level + L to fit a byte (Appendix F.1)."""
    hp = dict(beta1=0.9, beta2=0.99, lr=1e-4, wd=0.1, step=1)

    def pbit(W, p):
        z = np.ones((W, 4), np.float32)
        return orc.step_pbit(np.zeros(4, np.float32), z, z, p=p, **hp)

    def l1(W, L):
        z = np.zeros((W, 4), np.float32)
        z[:, 0] = 1.0                                               # four times the mean: clamped to the top level
        return orc.step_l1(np.zeros(4, np.float32), z, z, L=L, **hp)

    for W, p in ((1, 1), (3, 2), (15, 4), (127, 7), (255, 8)):
        assert pbit(W, p)["K"].tolist() == [W] * 4
    for W, p in ((2, 1), (4, 2), (16, 4), (128, 7), (1, 0), (1, 9), (256, 9)):
        with pytest.raises(orc.OracleError) as e:
            pbit(W, p)
        assert e.value.code == orc.ERR_RANGE
    for W, L in ((8, 15), (1, 127), (127, 1), (5, 25)):
        assert l1(W, L)["K"].tolist() == [2 * L * W] + [L * W] * 3  # bytes level + L: top level, then level 0
    for W, L in ((9, 15), (2, 64), (128, 1), (64, 2)):
        with pytest.raises(orc.OracleError) as e:
            l1(W, L)
        assert e.value.code == orc.ERR_RANGE


@pytest.mark.parametrize("W", [4, 8, 16, 64])
def test_tie_rate_closed_form_and_table3(W):
    """Independent fair signs tie with probability C(W, W/2) / 2^W; Table 3's measured
    tie rates on real gradients (4 and 8 workers) lie within half a point of that."""
    n = 1 << 20
    rng = np.random.default_rng(1234 + W)
    bits = rng.integers(0, 2, size=(W, n), dtype=np.uint8)
    K, S, u = orc.count_sign(bits, 1, orc.TIE_ZERO)
    rate = float(np.mean(u == 0))
    p = math.comb(W, W // 2) / 2.0 ** W
    sigma = math.sqrt(p * (1 - p) / n)
    assert abs(rate - p) < 5 * sigma
    gold = read_golden("paper_printed_values.txt")
    key = "table3.tie_pct.w%d" % W
    if key in gold:
        paper = sum(float(x) for x in gold[key].split("+")) / 100.0
        assert abs(rate - paper) < 0.005


# --------------------------------------------------------------------------------------
# Algorithm 1 line 3: exact rational arithmetic, conventions, special cases
# --------------------------------------------------------------------------------------
def _dyadic(rng, n, bits=6, scale=2.0 ** -10):
    return (rng.integers(-(1 << bits), (1 << bits) + 1, size=n) * scale).astype(np.float32)


@pytest.mark.parametrize("beta1", [0.5, 0.75, 0.875, 0.9375, 0.0, 1.0])
def test_local_sign_exact_rational(beta1):
    """With dyadic beta1 and few-bit dyadic inputs every fp32 operation is exact, so
    the oracle's sign must equal the sign of the rational beta1*m + (1-beta1)*g."""
    rng = np.random.default_rng(7)
    n = 4000
    m, g = _dyadic(rng, n), _dyadic(rng, n)
    # force exact cancellations and zeros into the sample
    if 0.0 < beta1 < 1.0:
        ratio = Fraction(beta1) / (1 - Fraction(beta1))
        m[:50] = _dyadic(rng, 50, bits=3)
        g[:50] = np.array([float(-ratio * Fraction(float(x))) for x in m[:50]], np.float32)
    m[50:60] = 0.0
    g[50:60] = 0.0
    s = orc.local_sign(m, g, beta1)
    b1 = Fraction(beta1)
    want = []
    for mi, gi in zip(m.tolist(), g.tolist()):
        c = b1 * Fraction(mi) + (1 - b1) * Fraction(gi)
        want.append((c > 0) - (c < 0))
    assert s.tolist() == want
    if 0.0 < beta1 < 1.0:
        assert (s[:60] == 0).all()
    assert orc.local_sign(m, g, beta1, exact=True).tolist() == want


def test_local_sign_fp32_pinned_order():
    """The sign is that of fma(beta1, m, fl32(fl32(1-beta1) * g)): rebuilt here with
    rationals and an explicit round-to-nearest-even to binary32."""
    rng = np.random.default_rng(11)
    n = 3000
    beta1 = np.float32(0.9)
    omb1 = np.float32(1.0) - beta1
    m = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    # near-cancellation: g chosen so that c is within a few ulps of zero
    g[:1000] = (-(beta1 * m[:1000]) / omb1).astype(np.float32)
    g[1000:1500] = np.nextafter(g[:500], np.float32(1.0))
    s = orc.local_sign(m, g, float(beta1))
    want = []
    for mi, gi in zip(m.tolist(), g.tolist()):
        t = Fraction(float(np.float32(Fraction(float(omb1)) * Fraction(gi))))  # one rounding
        c = Fraction(float(beta1)) * Fraction(mi) + t                          # fma: exact, then sign
        want.append((c > 0) - (c < 0))
    assert s.tolist() == want
    # the unrounded sign differs only where rounding t moved c across zero
    e = orc.local_sign(m, g, float(beta1), exact=True)
    assert np.mean(e[1500:] != s[1500:]) < 1e-3


def test_local_sign_fp32_vs_exact_on_gaussian():
    rng = np.random.default_rng(5)
    n = 1 << 20
    m = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    s = orc.local_sign(m, g, 0.9)
    e = orc.local_sign(m, g, 0.9, exact=True)
    assert int(np.sum(s != e)) <= 3
    assert int(np.sum(s == 0)) == 0          # standard Lion never outputs 0 (Table 3, last row)
    assert abs(float(np.mean(s > 0)) - 0.5) < 0.01


def test_sign_is_a_comparison_not_the_sign_bit():
    tiny = 2.0 ** -148                                   # twice the smallest denormal
    m = np.array([0.0, -0.0, np.nan, np.inf, -np.inf, tiny, -tiny, 0.0], np.float32)
    g = np.array([0.0, -0.0, 1.0, 1.0, 1.0, 0.0, 0.0, -0.0], np.float32)
    s = orc.local_sign(m, g, 0.5)
    assert s.tolist() == [0, 0, 0, 1, -1, 1, -1, 0]      # denormals keep their sign


def test_w1_is_textbook_lion_in_both_conventions():
    """One worker: the vote is the worker's own sign, so a step is plain Lion.  Section 2
    writes Lion with the momentum negated (m <- b2 m - (1-b2) g, theta <- theta +
    eta sign(b1 m - (1-b1) g)); Algorithm 1 accumulates +g and steps against the sign.
    Both give the same trajectory.  Exact rationals, dyadic hyper-parameters."""
    rng = np.random.default_rng(3)
    n, steps = 64, 6
    b1, b2, lr, wd = 0.75, 0.875, 2.0 ** -6, 0.0
    theta = _dyadic(rng, n)
    m = np.zeros((1, n), np.float32)
    th_ref = [Fraction(float(x)) for x in theta]
    mneg = [Fraction(0)] * n                                  # Section 2's momentum (= -m)
    for t in range(1, steps + 1):
        g = _dyadic(rng, n, bits=4, scale=2.0 ** -6)
        g[g == 0] = 2.0 ** -6                                 # keep c away from exact zero ...
        r = orc.step_1bit(theta, m, g[None], beta1=b1, beta2=b2, lr=lr, wd=wd, step=t)
        for i in range(n):
            gi = Fraction(float(g[i]))
            c = Fraction(b1) * mneg[i] - (1 - Fraction(b1)) * gi
            sg = (c > 0) - (c < 0)
            if sg == 0:                                       # ... else follow the zero rule
                sg = -1 if t % 2 == 1 else 1
            th_ref[i] = th_ref[i] + Fraction(lr) * sg
            mneg[i] = Fraction(b2) * mneg[i] - (1 - Fraction(b2)) * gi
        assert [Fraction(x) for x in r["theta"].tolist()] == th_ref
        assert [Fraction(x) for x in r["m"][0].tolist()] == [-x for x in mneg]
        theta = r["theta"].astype(np.float32)
        m = r["m"].astype(np.float32)
        assert [Fraction(float(x)) for x in theta] == th_ref  # still exact in fp32


def test_beta1_equals_beta2_is_sign_of_new_momentum():
    """Section 2: with beta1 = beta2 Lion is sign descent on the momentum -- the
    interpolation of line 3 is the new momentum of line 6."""
    rng = np.random.default_rng(9)
    n = 5000
    m, g = _dyadic(rng, n), _dyadic(rng, n)
    for beta in (0.5, 0.875):
        s = orc.local_sign(m, g, beta)
        mn = orc.momentum(m, g, beta)
        assert s.tolist() == np.sign(mn).astype(int).tolist()


def test_bf16_widening_matches_library_on_all_patterns():
    h = np.arange(65536, dtype=np.uint16)
    ref = torch.from_numpy(h.view(np.int16).copy()).view(torch.bfloat16).to(torch.float32).numpy()
    got = np.array([orc.bf16_to_f32(int(x)) for x in h], np.float32)
    nan = np.isnan(ref)                      # NaN payloads do not survive the trip through a Python float
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got.view(np.uint32)[~nan], ref.view(np.uint32)[~nan])
    assert np.array_equal(ref.view(np.uint32)[~nan], h.astype(np.uint32)[~nan] << 16)
    # and through the gradient argument: m = 0, beta1 = 0 -> sign(c) = sign(g)
    finite = ~np.isnan(ref)
    s = orc.local_sign(np.zeros(65536, np.float32), h, 0.0, g_dtype=orc.BF16)
    assert s[finite].tolist() == np.sign(ref[finite]).astype(int).tolist()
    assert (s[~finite] == 0).all()
    mn = orc.momentum(np.zeros(65536, np.float32), h, 0.0, g_dtype=orc.BF16)
    assert np.array_equal(mn[finite], ref[finite].astype(np.float64))


# --------------------------------------------------------------------------------------
# zero rule (Appendix B.1)
# --------------------------------------------------------------------------------------
def test_zero_rule_alternates_and_error_accumulates():
    """A parameter whose gradient is always zero (an unused position-embedding row)
    has c = 0 on every worker: iteration 1 votes it +1, iteration 2 votes it -1."""
    n, W = 70, 4
    z = np.zeros((W, n), np.float32)
    theta = np.full(n, 0.5, np.float32)
    hp = dict(beta1=0.9, beta2=0.99, lr=2.0 ** -7, wd=0.0)
    r1 = orc.step_1bit(theta, z, z, step=1, **hp)
    assert (r1["b"] == 1).all() and (r1["u"] == 1).all() and (r1["K"] == W).all()
    assert r1["words"][0].tolist() == [2 ** 64 - 1, 2 ** 6 - 1]          # pad bits are zero
    r2 = orc.step_1bit(r1["theta"].astype(np.float32), z, z, step=2, **hp)
    assert (r2["b"] == 0).all() and (r2["u"] == -1).all() and (r2["K"] == 0).all()
    assert np.array_equal(r2["theta"], theta.astype(np.float64))        # +lr then -lr
    s = np.array([1, 0, -1, 0], np.int8)
    assert orc.zero_rule(s, 1).tolist() == [1, 1, 0, 1]
    assert orc.zero_rule(s, 2).tolist() == [1, 0, 0, 0]
    assert orc.zero_rule(s, 2 ** 40 + 1).tolist() == [1, 1, 0, 1]
    assert orc.zero_rule(s, 2, orc.ZERO_POS).tolist() == [1, 1, 0, 1]
    assert orc.zero_rule(s, 1, orc.ZERO_NEG).tolist() == [1, 0, 0, 0]


# --------------------------------------------------------------------------------------
# packing
# --------------------------------------------------------------------------------------
@pytest.mark.parametrize("n", list(range(0, 200)) + [4095, 4096, 4097])
def test_pack_unpack_1bit_roundtrip(n):
    rng = np.random.default_rng(n)
    b = rng.integers(0, 2, n, dtype=np.uint8)
    words = orc.pack_1bit(b)
    assert words.size == (n + 63) // 64
    assert np.array_equal(orc.unpack_1bit(words, n), b)
    as_int = sum(int(x) << i for i, x in enumerate(b.tolist()))          # LSB-first big integer
    assert sum(int(w) << (64 * j) for j, w in enumerate(words.tolist())) == as_int
    assert sum(bin(int(w)).count("1") for w in words) == int(b.sum())


@pytest.mark.parametrize("p", range(1, 9))
@pytest.mark.parametrize("n", [0, 1, 2, 3, 7, 8, 9, 63, 64, 65, 130])
def test_pack_unpack_fields_roundtrip(p, n):
    C = orc.container_bits(p)
    assert C == {1: 1, 2: 2, 3: 4, 4: 4, 5: 8, 6: 8, 7: 8, 8: 8}[p]   # 7 bits take a byte
    rng = np.random.default_rng(100 * p + n)
    v = rng.integers(0, 1 << C, n, dtype=np.uint8)
    by = orc.pack_fields(v, p)
    assert by.size == (n * C + 7) // 8
    assert np.array_equal(orc.unpack_fields(by, n, p), v)
    as_int = sum(int(x) << (C * i) for i, x in enumerate(v.tolist()))
    assert int.from_bytes(by.tobytes(), "little") == as_int
    if C == 1:
        w = orc.pack_1bit(v)
        assert w.tobytes()[:by.size] == by.tobytes()      # same bit order as the 1-bit words


def test_fields_reject_bad_width_and_overflowing_value():
    for p in (0, 9, -1):
        assert orc.container_bits(p) == -1
        with pytest.raises(orc.OracleError):
            orc.pack_fields(np.zeros(4, np.uint8), p)
    with pytest.raises(orc.OracleError):
        orc.pack_fields(np.array([16], np.uint8), 4)


# --------------------------------------------------------------------------------------
# aggregation: brute force, invariants, two independent formulations
# --------------------------------------------------------------------------------------
@pytest.mark.parametrize("W", range(1, 13))
def test_vote_brute_force_all_bit_columns(W):
    cols = np.array(list(itertools.product([0, 1], repeat=W)), np.uint8).T.copy()   # (W, 2^W)
    for step in (1, 2):
        for tie in (orc.TIE_ZERO, orc.TIE_ALT):
            K, S, u = orc.count_sign(cols, step, tie)
            for j in range(cols.shape[1]):
                signs = [2 * int(x) - 1 for x in cols[:, j]]
                tot = sum(signs)
                want = (tot > 0) - (tot < 0)
                if want == 0 and tie == orc.TIE_ALT:
                    want = 1 if step % 2 == 1 else -1
                assert (K[j], S[j], u[j]) == (sum(int(x) for x in cols[:, j]), tot, want)
            assert (np.abs(S) <= W).all() and ((S - W) % 2 == 0).all()
            assert (K >= 0).all() and (K <= W).all()
            if W % 2 == 1:
                assert (u != 0).all()


@pytest.mark.parametrize("W", range(1, 8))
def test_vote_brute_force_all_ternary_columns(W):
    """All 3^W columns of worker signs through zero rule -> vote, against the sum of
    the forced signs done with Python integers."""
    cols = np.array(list(itertools.product([-1, 0, 1], repeat=W)), np.int8).T.copy()
    n = cols.shape[1]
    for step in (1, 2):
        z = 1 if step % 2 == 1 else -1
        b = np.stack([orc.zero_rule(cols[w], step) for w in range(W)])
        K, S, u = orc.count_sign(b, step, orc.TIE_ZERO)
        for j in range(n):
            forced = [int(x) if x != 0 else z for x in cols[:, j]]
            tot = sum(forced)
            assert S[j] == tot and u[j] == (tot > 0) - (tot < 0)


@pytest.mark.parametrize("W,p", [(3, 2), (8, 4), (15, 4), (64, 7), (125, 8), (255, 8), (1, 1)])
def test_field_sum_equals_bit_count(W, p):
    """K from summing packed p-bit containers byte-wise (what the summing allreduce
    does) = K from counting bits = column sums; total of K = total popcount."""
    n = 777
    rng = np.random.default_rng(W * 10 + p)
    b = rng.integers(0, 2, (W, n), dtype=np.uint8)
    b[:, :5] = 1                                            # K = W must survive the field width
    b[:, 5:9] = 0
    fields = np.stack([orc.pack_fields(b[w], p) for w in range(W)])
    K8 = orc.unpack_fields(orc.sum_bytes(fields), n, p)
    K, S, u = orc.count_sign(b, 1, p=p)
    assert np.array_equal(K8.astype(np.int32), K)
    assert np.array_equal(K, b.astype(np.int64).sum(0))
    words = [orc.pack_1bit(b[w]) for w in range(W)]
    assert int(K.sum()) == sum(bin(int(x)).count("1") for w in words for x in w)
    assert K[:5].tolist() == [W] * 5 and K[5:9].tolist() == [0] * 4
    with pytest.raises(orc.OracleError):
        orc.count_sign(np.ones((1 << p, 2), np.uint8), 1, p=p)   # W = 2^p is one too many


def test_planes_roundtrip_and_layout():
    rng = np.random.default_rng(21)
    for n in (1, 63, 64, 65, 1000):
        u = rng.integers(-1, 2, n).astype(np.int8)
        pos, nz = orc.planes(u)
        assert np.array_equal(orc.unplanes(pos, nz, n), u)
        assert np.array_equal(pos, orc.pack_1bit((u > 0).astype(np.uint8)))
        assert np.array_equal(nz, orc.pack_1bit((u != 0).astype(np.uint8)))
        assert not (pos & ~nz).any()


# --------------------------------------------------------------------------------------
# apply, momentum, averaging: closed forms and special cases
# --------------------------------------------------------------------------------------
def test_apply_closed_form_values():
    gold = read_golden("apply_closed_form.txt")
    th, lr, wd = np.float32(gold["theta"]), np.float32(gold["lr"]), np.float32(gold["wd"])
    out = orc.apply(np.array([th] * 3), np.array([1, 0, -1], np.int8), float(lr), float(wd))
    want = [float(gold["out.plus"]), float(gold["out.zero"]), float(gold["out.minus"])]
    # inputs are the fp32 neighbours of the decimals: 1e-7 relative covers that
    assert np.allclose(out, want, rtol=2e-7, atol=0)
    exact = [Fraction(float(th)) - Fraction(float(lr)) * (u + Fraction(float(wd)) * Fraction(float(th)))
             for u in (1, 0, -1)]
    assert np.allclose(out, [float(x) for x in exact], rtol=1e-15, atol=0)


def test_apply_special_cases():
    rng = np.random.default_rng(2)
    n = 1000
    theta = (rng.standard_normal(n) * 0.02).astype(np.float32)
    u = rng.integers(-1, 2, n).astype(np.int8)
    assert np.array_equal(orc.apply(theta, u, 0.0, 0.1), theta.astype(np.float64))      # lr = 0
    d = orc.apply(theta, u, 2.0 ** -10, 0.0) - theta                                   # wd = 0
    assert np.array_equal(d, -(2.0 ** -10) * u)
    shr = orc.apply(theta, np.zeros(n, np.int8), 0.25, 0.5)                            # pure decay
    assert np.array_equal(shr, theta.astype(np.float64) * (1 - 0.125))
    # moves against the vote: +1 lowers theta, -1 raises it
    up = orc.apply(theta, np.ones(n, np.int8), 1e-3, 0.0)
    assert (up < theta).all()


def test_momentum_closed_forms():
    rng = np.random.default_rng(4)
    n = 500
    m = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    assert np.array_equal(orc.momentum(m, g, 1.0), m.astype(np.float64))     # beta2 = 1
    assert np.array_equal(orc.momentum(m, g, 0.0), g.astype(np.float64))     # beta2 = 0
    half = orc.momentum(m, g, 0.5)
    assert np.array_equal(half, (m.astype(np.float64) + g) / 2)
    # constant gradient from m0 = 0: m_t = (1 - beta2^t) g   (geometric series)
    b2 = float(np.float32(0.99))
    mt = np.zeros(n, np.float64)
    for t in range(1, 21):
        mt = orc.momentum(mt.astype(np.float32), g, 0.99)
        assert np.allclose(mt, (1 - b2 ** t) * g.astype(np.float64), rtol=1e-5, atol=1e-12)
    # beta2 = 0.99 weighs the old momentum, not the gradient
    assert np.allclose(orc.momentum(np.ones(1, np.float32), np.zeros(1, np.float32), 0.99), b2)


def test_momentum_avg():
    rng = np.random.default_rng(6)
    W, n = 5, 300
    m = _dyadic(rng, W * n, bits=10).reshape(W, n)
    mean = orc.momentum_avg(m)
    want = [sum(Fraction(float(m[w, i])) for w in range(W)) / W for i in range(n)]
    assert np.allclose(mean, [float(x) for x in want], rtol=1e-15, atol=0)
    same = np.repeat(m[:1], W, 0)
    assert np.array_equal(orc.momentum_avg(same), m[0].astype(np.float64))    # identical -> unchanged
    assert np.allclose(mean * W, m.astype(np.float64).sum(0), rtol=1e-15)     # the sum is preserved
    # one worker differs: the mean moves by delta / W, not delta
    m2 = same.copy()
    m2[3] += np.float32(0.5)
    assert np.allclose(orc.momentum_avg(m2) - m[0], 0.5 / W, rtol=1e-12)


# --------------------------------------------------------------------------------------
# whole step, tiny, against an independent exact re-derivation in rationals
# --------------------------------------------------------------------------------------
@pytest.mark.parametrize("W,n,step", [(1, 5, 1), (2, 64, 2), (3, 65, 1), (4, 130, 2), (5, 33, 3)])
def test_whole_step_brute_force_rationals(W, n, step):
    rng = np.random.default_rng(1000 + W)
    b1, b2, lr, wd = 0.875, 0.9375, 2.0 ** -8, 0.125
    theta = _dyadic(rng, n)
    m = _dyadic(rng, W * n, bits=3).reshape(W, n)
    g = _dyadic(rng, W * n, bits=3).reshape(W, n)
    g[:, : n // 4] = (-7 * m[:, : n // 4]).astype(np.float32)      # c = 0 exactly there
    r = orc.step_1bit(theta, m, g, beta1=b1, beta2=b2, lr=lr, wd=wd, step=step)
    rp = orc.step_pbit(theta, m, g, p=3, beta1=b1, beta2=b2, lr=lr, wd=wd, step=step)
    z = 1 if step % 2 == 1 else -1
    big = [0] * W
    for i in range(n):
        tot = 0
        for w in range(W):
            c = Fraction(b1) * Fraction(float(m[w, i])) + (1 - Fraction(b1)) * Fraction(float(g[w, i]))
            sg = (c > 0) - (c < 0)
            assert r["s"][w, i] == sg
            sg = sg if sg else z
            big[w] |= (1 if sg > 0 else 0) << i
            tot += sg
            mn = Fraction(b2) * Fraction(float(m[w, i])) + (1 - Fraction(b2)) * Fraction(float(g[w, i]))
            assert Fraction(float(r["m"][w, i])) == mn
        uu = (tot > 0) - (tot < 0)
        assert r["u"][i] == uu and rp["u"][i] == uu and rp["K"][i] == (tot + W) // 2
        th = Fraction(float(theta[i]))
        assert Fraction(float(r["theta"][i])) == th - Fraction(lr) * (uu + Fraction(wd) * th)
    for w in range(W):
        assert sum(int(x) << (64 * j) for j, x in enumerate(r["words"][w].tolist())) == big[w]
    assert (r["s"][:, : n // 4] == 0).all()
    assert np.array_equal(r["theta"], rp["theta"]) and np.array_equal(r["pos"], rp["pos"])


# --------------------------------------------------------------------------------------
# ternary wire format (Appendix B.1): exact zeros travel, the vote is the sign of the sum
# --------------------------------------------------------------------------------------
@pytest.mark.parametrize("W", range(1, 8))
def test_ternary_vote_brute_force(W):
    cols = np.array(list(itertools.product([-1, 0, 1], repeat=W)), np.int8).T.copy()     # all 3^W columns
    Kp, Kn, S, u = orc.ternary_vote(cols)
    for j in range(cols.shape[1]):
        col = [int(x) for x in cols[:, j]]
        tot = sum(col)
        assert (Kp[j], Kn[j], S[j], u[j]) == (col.count(1), col.count(-1), tot, (tot > 0) - (tot < 0))
    assert (Kp + Kn <= W).all()


def test_ternary_hand_case_and_difference_to_one_bit(hand):
    """The hand case's last element has gradient 0 on every worker: the 1-bit path votes
    it +1 or -1 by iteration parity, the ternary format keeps it 0 (what Appendix B.1's
    2-bit allreduce transmits).  Elsewhere, without zeros, both agree."""
    gold, g = hand
    theta = np.zeros(8, np.float32)
    m = np.zeros((3, 8), np.float32)
    r = orc.step_ternary(theta, m, g[:3], beta1=0.9, beta2=0.99, lr=1e-4, wd=0.0)
    assert r["S"].tolist() == _ints(gold["step1.W3.S"])[:7] + [0]
    assert r["u"].tolist() == [1, -1, -1, -1, 1, -1, 1, 0]
    assert [int(r["pos"][0]), int(r["nz"][0])] == [0x51, 0x7F]
    assert [int(x) for x in r["pos_w"][:, 0]] == [0x53, 0x19, 0x45]          # = the even-iteration 1-bit words
    assert [int(x) for x in r["nz_w"][:, 0]] == [0x7F, 0x7F, 0x7F]
    one = orc.step_1bit(theta, m, g[:3], beta1=0.9, beta2=0.99, lr=1e-4, wd=0.0, step=1)
    assert one["u"][:7].tolist() == r["u"][:7].tolist() and one["u"][7] == 1 and r["u"][7] == 0
    r4 = orc.step_ternary(theta, np.zeros((4, 8), np.float32), g, beta1=0.9, beta2=0.99, lr=1e-4, wd=0.0)
    assert r4["S"].tolist() == _ints(gold["step1.W4.S"])[:7] + [0]           # ties stay 0 by themselves


# --------------------------------------------------------------------------------------
# divergence metric of Section 5.1 (max over elements of the std across workers)
# --------------------------------------------------------------------------------------
def test_momentum_divergence_closed_forms():
    rng = np.random.default_rng(17)
    n = 400
    a = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    b = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    # two workers: the std of {a, b} is |a - b| / 2
    want = float(np.max(np.abs(a.astype(np.float64) - b) / 2))
    assert orc.momentum_divergence(np.stack([a, b])) == pytest.approx(want, rel=1e-14)
    assert orc.momentum_divergence(np.stack([a, a, a])) == 0.0                   # synchronised momenta
    for W in (3, 8, 16):
        m = (rng.standard_normal((W, n)) * 1e-3).astype(np.float32)
        lib = float(np.max(np.std(m.astype(np.float64), axis=0)))              # library routine, ddof = 0
        assert orc.momentum_divergence(m) == pytest.approx(lib, rel=1e-12)
        assert orc.momentum_divergence(m * np.float32(4.0)) == pytest.approx(4 * lib, rel=1e-12)
        shifted = m + np.float32(1.0)                                           # a common offset changes nothing
        assert orc.momentum_divergence(shifted) == pytest.approx(
            float(np.max(np.std(shifted.astype(np.float64), axis=0))), rel=1e-9)
    # one element stands out: it alone sets the maximum ({0,0,0,1}: mean 1/4, std sqrt(3)/4)
    m = np.zeros((4, 50), np.float32)
    m[3, 7] = 1.0
    assert orc.momentum_divergence(m) == pytest.approx(math.sqrt(3) / 4, rel=1e-15)
    # averaging the momenta (Section 5) removes the divergence
    avg = orc.momentum_avg(m).astype(np.float32)
    assert orc.momentum_divergence(np.repeat(avg[None], 4, 0)) == 0.0
    # the maximum may sit at either end of the range
    for at in (0, 49):
        m = np.zeros((4, 50), np.float32)
        m[1, at] = 2.0
        assert orc.momentum_divergence(m) == pytest.approx(math.sqrt(3) / 2, rel=1e-15)


def test_oracle_loops_write_nothing_outside_their_outputs():
    """Every C loop of the oracle is called on a ragged length with its outputs cut out of
    larger arrays of a marker byte: the bytes on either side must keep the marker."""
    for n in (67, 64 * 63):
        _guard_band_pass(n)


def _guard_band_pass(n):
    W, guard, mark = 3, 64, 0xA5
    rng = np.random.default_rng(23)
    checks = []

    def out(count, dtype):
        raw = np.full(count * np.dtype(dtype).itemsize + 2 * guard, mark, np.uint8)
        checks.append((raw, count * np.dtype(dtype).itemsize))
        return raw[guard:guard + count * np.dtype(dtype).itemsize].view(dtype)

    ptr = orc._p
    m = rng.standard_normal((W, n)).astype(np.float32)
    g = rng.standard_normal((W, n)).astype(np.float32)
    gb = (g.view(np.uint32) >> 16).astype(np.uint16)
    nw = orc.n_words(n)
    s = out(n, np.int8)
    orc._local_sign(ptr(m[0]), ptr(g[0]), orc.F32, n, 0.9, ptr(s))
    orc._local_sign_exact(ptr(m[0]), ptr(gb[0]), orc.BF16, n, 0.9, ptr(out(n, np.int8)))
    b = out(n, np.uint8)
    orc._zero_rule(ptr(s), n, 1, orc.ZERO_ALT, ptr(b))
    words = out(nw, np.uint64)
    orc._pack_1bit(ptr(b), n, ptr(words))
    orc._unpack_1bit(ptr(words), n, ptr(out(n, np.uint8)))
    for p in (2, 3, 4, 8):
        fields = out(orc.field_bytes(n, p), np.uint8)
        assert orc._pack_fields(ptr(b), n, p, ptr(fields)) == 0
        assert orc._unpack_fields(ptr(fields), n, p, ptr(out(n, np.uint8))) == 0
    bits = rng.integers(0, 2, (W, n)).astype(np.uint8)
    u = out(n, np.int8)
    assert orc._count_sign(ptr(bits), W, n, 0, 1, orc.TIE_ZERO, ptr(out(n, np.int32)), ptr(out(n, np.int32)), ptr(u)) == 0
    pos, nz = out(nw, np.uint64), out(nw, np.uint64)
    orc._planes(ptr(u), n, ptr(pos), ptr(nz))
    orc._unplanes(ptr(pos), ptr(nz), n, ptr(out(n, np.int8)))
    orc._apply(ptr(m[0]), ptr(u), n, 1e-4, 0.1, ptr(out(n, np.float64)))
    orc._momentum(ptr(m[0]), ptr(g[0]), orc.F32, n, 0.99, ptr(out(n, np.float64)))
    orc._momentum_avg(ptr(m), W, n, ptr(out(n, np.float64)))
    orc._sum_bytes(ptr(bits), W, n, ptr(out(n, np.uint8)))
    c = out(n, np.float32)
    orc._local_c(ptr(m[0]), ptr(g[0]), orc.F32, n, 0.9, ptr(c))
    totals = out(256, np.uint64)                           # arrives full of the marker: the function clears it itself
    orc._abs_totals(ptr(c), n, ptr(totals))
    clean = np.zeros(256, np.uint64)
    orc._abs_totals(ptr(c), n, ptr(clean))
    assert np.array_equal(totals, clean) and clean.sum() > 0
    lev = out(n, np.int8)
    orc._l1_levels(ptr(c), n, orc.mean_abs(c), 15, ptr(lev))
    rows = (rng.integers(-15, 16, (W, n)) + 15).astype(np.uint8)
    assert orc._level_sum_sign(ptr(rows), W, n, 15, 1, orc.TIE_ZERO, ptr(out(n, np.int32)), ptr(out(n, np.int32)), ptr(out(n, np.int8))) == 0
    tern = rng.integers(-1, 2, (W, n)).astype(np.int8)
    assert orc._ternary_vote(ptr(tern), W, n, ptr(out(n, np.int32)), ptr(out(n, np.int32)), ptr(out(n, np.int32)), ptr(out(n, np.int8))) == 0
    assert len(checks) >= 30
    for raw, size in checks:
        assert np.all(raw[:guard] == mark) and np.all(raw[guard + size:] == mark)
