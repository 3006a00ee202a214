"""Pins for the oracle's L1 quantisation (Equation 1 with p = 1; Appendix F.1): the
hand-worked case, the exact mean against the standard library's correctly rounded sum,
algebraic properties of Equation 1, and brute force with rationals.  No GPU needed."""
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle as orc
from conftest import read_golden


def _nums(s, conv=float):
    return [conv(v) for v in s.split()]


def test_hand_case():
    g = read_golden("l1_hand_case.txt")
    x = np.array(_nums(g["x"]), np.float32)
    L = int(g["L"])
    M = orc.mean_abs(x)
    assert M == float(g["mean_abs"])
    lv = orc.l1_levels(x, M, L)
    assert lv.tolist() == _nums(g["levels"], int)
    by = (lv.astype(np.int16) + L).astype(np.uint8)
    assert by.tolist() == _nums(g["bytes"], int)
    rows = np.stack([by, (2 * L - by.astype(np.int16)).astype(np.uint8), by])      # x, -x, x
    K, S, u = orc.level_sum_sign(rows, L, 1)
    assert K.tolist() == _nums(g["sum3.K"], int) and S.tolist() == _nums(g["sum3.S"], int)
    assert u.tolist() == _nums(g["sum3.u"], int)
    wmax = int(g["L15.max_workers"])
    orc.level_sum_sign(np.repeat(by[None], wmax, 0), L, 1)
    with pytest.raises(orc.OracleError) as e:
        orc.level_sum_sign(np.repeat(by[None], wmax + 1, 0), L, 1)
    assert e.value.code == orc.ERR_RANGE
    # the whole step through Algorithm 1: beta1 = 0 and m = 0 make c = g exactly
    r = orc.step_l1(np.zeros(8, np.float32), np.zeros((3, 8), np.float32), np.stack([x, -x, x]), L=L, beta1=0.0,
                    beta2=0.5, lr=2.0 ** -6, wd=0.0, step=1)
    assert r["S"].tolist() == _nums(g["sum3.S"], int)
    assert np.array_equal(r["theta"], -(2.0 ** -6) * np.array(_nums(g["sum3.u"])))


@pytest.mark.parametrize("seed", range(6))
def test_mean_abs_is_the_correctly_rounded_exact_sum(seed):
    """Against math.fsum (exact sum, one rounding), on wide dynamic ranges, denormals,
    cancellation-free by construction (absolute values)."""
    rng = np.random.default_rng(seed)
    n = [1, 7, 1000, 4097, 20000, 65536][seed]
    x = (rng.standard_normal(n) * np.exp2(rng.integers(-140, 100, n))).astype(np.float32)
    x[rng.integers(0, n, max(1, n // 10))] = 0.0
    if n > 10:
        x[:4] = [2.0 ** -149, -(2.0 ** -140), 3.0e38, -1.0e-45]
    want = math.fsum(abs(float(v)) for v in x) / n
    assert orc.mean_abs(x) == want
    assert orc.mean_abs(np.zeros(5, np.float32)) == 0.0
    assert orc.mean_abs(np.zeros(0, np.float32)) == 0.0
    assert math.isnan(orc.mean_abs(np.array([1.0, np.inf], np.float32)))


def test_mean_abs_of_denormals_alone_is_exact():
    """Denormals carry no hidden bit and share the smallest exponent: a sum made of them
    alone, and of them beside the smallest normals, is a small integer times 2^-149."""
    tiny = 2.0 ** -149
    x = np.array([tiny, -3 * tiny, 5 * tiny, -(2.0 ** -127), 0.0, -0.0, 0.0, 0.0], np.float32)
    assert np.all(np.abs(x) < np.float32(2.0 ** -126))
    assert Fraction(orc.mean_abs(x)) == Fraction(1 + 3 + 5 + 2 ** 22, 8) * Fraction(1, 2 ** 149)
    y = np.array([2.0 ** -126, 7 * tiny, -(2.0 ** -125), -tiny], np.float32)      # two normals, two denormals
    assert Fraction(orc.mean_abs(y)) == Fraction(2 ** 23 + 7 + 2 ** 24 + 1, 4) * Fraction(1, 2 ** 149)
    rng = np.random.default_rng(5)
    z = (rng.integers(-(2 ** 23) + 1, 2 ** 23, 4096) * tiny).astype(np.float32)   # every denormal pattern is fair game
    assert Fraction(orc.mean_abs(z)) == Fraction(int(np.abs(np.round(z.astype(np.float64) / tiny)).sum()), 4096) / 2 ** 149


def test_mean_abs_does_not_depend_on_order_and_beats_naive_fp32():
    rng = np.random.default_rng(3)
    x = np.concatenate([np.full(1, 2.0 ** 24, np.float32), np.ones(1 << 16, np.float32)])
    M = orc.mean_abs(x)
    assert M == (2.0 ** 24 + 2.0 ** 16) / x.size                # fp32 running sum would lose every 1.0
    assert orc.mean_abs(rng.permutation(x)) == M


@pytest.mark.parametrize("L", [1, 3, 7, 15, 127])
def test_equation1_against_rationals(L):
    """Dyadic inputs whose scaled values are exact in fp32: level = clamp(round-half-even(L x / (2 M)))."""
    rng = np.random.default_rng(L)
    n = 512
    j = {1: 3, 3: 5, 7: 6, 15: 7, 127: 10}[L]
    M_target = Fraction(L, 2 ** j)                               # then L / (2 M_1) = 2^(j-1): a dyadic scale
    x = (rng.integers(-48, 49, n) * 2.0 ** -8).astype(np.float32)
    rest = n * M_target - sum(Fraction(float(abs(v))) for v in x[1:])
    assert rest > 0
    x[0] = np.float32(float(rest))                               # one large entry makes the mean exact
    assert Fraction(float(x[0])) == rest
    M = orc.mean_abs(x)
    assert Fraction(M) == M_target
    got = orc.l1_levels(x, M, L).tolist()
    scale = Fraction(L) / (2 * M_target)
    assert scale == 2 ** (j - 1)
    halves = 0
    for v, lv in zip(x.tolist(), got):
        t = scale * Fraction(v)                                  # exact in fp32: multiples of 2^(j-9)
        halves += (t.denominator == 2)
        r = round(t)                                             # Python rounds exact halves to even
        assert lv == max(-L, min(L, r))
    assert halves > 0 or j > 8                                   # exact .5 cases occur where the grid allows
    assert max(got) <= L and min(got) >= -L


def test_equation1_properties():
    rng = np.random.default_rng(8)
    n, L = 10000, 15
    x = (rng.laplace(size=n) * 1e-3).astype(np.float32)
    M = orc.mean_abs(x)
    lv = orc.l1_levels(x, M, L)
    assert np.array_equal(orc.l1_levels(-x, M, L), -lv)                              # odd function
    for k in (-20, 7):                                                               # scale invariance
        xs = np.ldexp(x, k).astype(np.float32)
        assert np.array_equal(orc.l1_levels(xs, orc.mean_abs(xs), L), lv)
    assert (np.abs(lv[np.abs(x) >= 2 * M * (1 + 1e-6)]) == L).all()                  # clamp beyond 2 M_1
    assert (lv[np.abs(x) < M / L * (1 - 1e-6)] == 0).all()                           # |scale x| < 1/2 -> 0
    assert (np.sign(lv) * np.sign(x) >= 0).all()                                     # never flips a sign
    c = np.full(64, -0.5, np.float32)                       # constant vector: M_1 = |a| = 0.5, scale = L exactly
    assert set(orc.l1_levels(c, orc.mean_abs(c), 15).tolist()) == {-8}               # round(7.5) -> 8 (half to even)
    assert set(orc.l1_levels(c, orc.mean_abs(c), 7).tolist()) == {-4}                # round(3.5) -> 4
    assert set(orc.l1_levels(c, orc.mean_abs(c), 3).tolist()) == {-2}                # round(1.5) -> 2
    assert set(orc.l1_levels(np.zeros(9, np.float32), 0.0, 15).tolist()) == {0}
    # outliers do not wipe out the bulk, unlike max-norm scaling (Section 4.1)
    y = x.copy()
    y[0] = 1.63
    frac_zero = float(np.mean(orc.l1_levels(y, orc.mean_abs(y), L) == 0))
    assert frac_zero < 0.2


@pytest.mark.parametrize("W,L", [(1, 127), (2, 63), (4, 31), (8, 15), (17, 7), (127, 1)])
def test_level_sum_brute_force(W, L):
    rng = np.random.default_rng(W)
    n = 300
    lv = rng.integers(-L, L + 1, (W, n))
    lv[:, :3] = L
    lv[:, 3:6] = -L
    rows = (lv + L).astype(np.uint8)
    for step in (1, 2):
        for tie in (orc.TIE_ZERO, orc.TIE_ALT):
            K, S, u = orc.level_sum_sign(rows, L, step, tie)
            tot = lv.sum(0)
            want = np.sign(tot)
            if tie == orc.TIE_ALT:
                want[tot == 0] = 1 if step % 2 else -1
            assert np.array_equal(S, tot) and np.array_equal(K, tot + W * L) and np.array_equal(u, want)
            assert K.max() <= 255 and K[:3].tolist() == [2 * L * W] * 3 and K[3:6].tolist() == [0] * 3
    with pytest.raises(orc.OracleError):
        orc.level_sum_sign(np.zeros((W + 1 if 2 * L * (W + 1) > 255 else 200, n), np.uint8), L, 1)


def test_l1_with_one_level_is_not_the_sign():
    """With L = 1 (2 bits) values below M_1 in magnitude quantise to 0: richer than 1 bit
    only through the zero level -- and the vote over levels equals the majority vote
    whenever every |c| exceeds M_1 ... which a mean never allows for all entries."""
    x = np.array([3.0, -3.0, 0.9, -0.9, 1.0, 1.1], np.float32)
    M = orc.mean_abs(x)                                          # 1.65
    assert orc.l1_levels(x, M, 1).tolist() == [1, -1, 0, 0, 0, 0]


def _round_to_binary32(q):
    """A rational rounded once to the nearest binary32 (ties to even), as a Fraction; the
    inputs here stay inside the normal range, where numpy's float64 -> float32 conversion
    after an exact float64 representation would round twice, so the rounding is done by hand."""
    if q == 0:
        return Fraction(0)
    sign = -1 if q < 0 else 1
    a = abs(q)
    e = a.numerator.bit_length() - a.denominator.bit_length()           # 2^e <= a < 2^(e+2) roughly
    while Fraction(2) ** e > a:
        e -= 1
    while Fraction(2) ** (e + 1) <= a:
        e += 1
    e = max(e, -126)                                                    # denormals share the exponent of 2^-126
    ulp = Fraction(2) ** (e - 23)
    k = a / ulp
    lo = k.numerator // k.denominator
    rem = k - lo
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and lo % 2 == 1):
        lo += 1
    return sign * lo * ulp


@pytest.mark.parametrize("beta1", [0.75, 0.9, 0.95])
def test_local_c_is_the_fma_of_the_rounded_product(beta1):
    """Algorithm 1 line 3 in the pinned fp32 order: c = fl32(beta1 * m + fl32(fl32(1 - beta1) * g)),
    the inner product rounded once, the sum of the exact product beta1 * m and that value
    rounded once (a fused multiply-add).  Rebuilt with rationals on ordinary and on
    near-cancelling inputs, with m != 0: a separate multiply and add, a swapped weight or an
    unrounded (1 - beta1) all give other bits here.  The sign of c is the sign the 1-bit
    path packs."""
    rng = np.random.default_rng(int(beta1 * 100))
    n = 1500
    b1 = np.float32(beta1)
    omb1 = np.float32(1.0) - b1
    m = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    g[:500] = (-(b1 * m[:500]) / omb1).astype(np.float32)               # c within a few ulps of zero
    g[500:750] = np.nextafter(g[:250], np.float32(1.0))
    g[750:760] = 0.0
    m[760:770] = 0.0
    c = orc.local_c(m, g, beta1)
    assert c.dtype == np.float32
    want = []
    for mi, gi in zip(m.tolist(), g.tolist()):
        t = _round_to_binary32(Fraction(float(omb1)) * Fraction(gi))
        want.append(_round_to_binary32(Fraction(float(b1)) * Fraction(mi) + t))
    assert [Fraction(float(v)) for v in c.tolist()] == want
    assert np.array_equal(np.sign(c).astype(np.int8), orc.local_sign(m, g, beta1))
    # what the planted mistakes would give differs on these inputs
    mul_add = (b1 * m).astype(np.float32) + (omb1 * g).astype(np.float32)
    assert np.any(mul_add.astype(np.float32) != c)
    swapped = orc.local_c(g, m, beta1)
    assert np.any(swapped != c)


def test_round_to_binary32_helper_matches_numpy_on_float64_inputs():
    """The helper against numpy's single rounding float64 -> float32."""
    rng = np.random.default_rng(1)
    x = rng.standard_normal(2000) * np.exp2(rng.integers(-100, 100, 2000))
    x[:4] = [2.0 ** -130, 1.0 + 2.0 ** -24, 1.0 + 3 * 2.0 ** -24, -(2.0 ** -127) * 1.5]
    for v in x.tolist():
        assert _round_to_binary32(Fraction(v)) == Fraction(float(np.float32(v)))
