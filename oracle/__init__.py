"""CPU oracle for the Lion Cub compressed-update hot path -- TEST INFRASTRUCTURE.

Thin numpy/ctypes front of ``lioncub_oracle.c`` (plain C, one element at a time, fp64
for real-valued outputs).  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package; the HIP library and its
Python binding never do, and nothing here imports them.

The wrappers only allocate outputs and marshal arguments.  ``step_1bit`` and
``step_pbit`` chain the C functions in the order of Algorithm 1 of the paper
(arXiv 2411.16462) and return every intermediate, so that a test can compare each
stage of the HIP path with it.
"""
import ctypes as C

import numpy as np

from . import build as _build

F32, BF16 = 0, 1
ZERO_ALT, ZERO_POS, ZERO_NEG = 0, 1, 2
TIE_ZERO, TIE_ALT = 0, 1
OK, ERR_RANGE, ERR_ARG = 0, 4, 7

_lib = C.CDLL(_build.build())

_vp, _sz, _i, _u64, _f = C.c_void_p, C.c_size_t, C.c_int, C.c_uint64, C.c_float


def _sig(name, res, *args):
    fn = getattr(_lib, name)
    fn.restype = res
    fn.argtypes = list(args)
    return fn


_bf16_to_f32 = _sig("orc_bf16_to_f32", C.c_float, C.c_uint16)
_local_sign = _sig("orc_local_sign", None, _vp, _vp, _i, _sz, _f, _vp)
_local_sign_exact = _sig("orc_local_sign_exact", None, _vp, _vp, _i, _sz, _f, _vp)
_zero_rule = _sig("orc_zero_rule", None, _vp, _sz, _u64, _i, _vp)
_pack_1bit = _sig("orc_pack_1bit", None, _vp, _sz, _vp)
_unpack_1bit = _sig("orc_unpack_1bit", None, _vp, _sz, _vp)
_container_bits = _sig("orc_container_bits", _i, _i)
_pack_fields = _sig("orc_pack_fields", _i, _vp, _sz, _i, _vp)
_unpack_fields = _sig("orc_unpack_fields", _i, _vp, _sz, _i, _vp)
_count_sign = _sig("orc_count_sign", _i, _vp, _i, _sz, _i, _u64, _i, _vp, _vp, _vp)
_planes = _sig("orc_planes", None, _vp, _sz, _vp, _vp)
_unplanes = _sig("orc_unplanes", None, _vp, _vp, _sz, _vp)
_apply = _sig("orc_apply", None, _vp, _vp, _sz, _f, _f, _vp)
_momentum = _sig("orc_momentum", None, _vp, _vp, _i, _sz, _f, _vp)
_momentum_avg = _sig("orc_momentum_avg", None, _vp, _i, _sz, _vp)
_sum_bytes = _sig("orc_sum_bytes", None, _vp, _i, _sz, _vp)


class OracleError(ValueError):
    def __init__(self, code, what):
        super().__init__("%s: oracle status %d" % (what, code))
        self.code = code


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _arr(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _grad(g, g_dtype):
    """fp32 gradients as float32, bf16 gradients as their raw uint16 bit patterns."""
    return _arr(g, np.uint16 if g_dtype == BF16 else np.float32)


def n_words(n):
    return (n + 63) // 64


def bf16_to_f32(h):
    return float(_bf16_to_f32(int(h)))


def local_sign(m, g, beta1, g_dtype=F32, exact=False):
    """Algorithm 1 line 3 and the sign: int8 array in {-1, 0, +1}."""
    m = _arr(m, np.float32)
    g = _grad(g, g_dtype)
    assert m.ndim == 1 and g.shape == m.shape
    s = np.empty(m.shape, np.int8)
    (_local_sign_exact if exact else _local_sign)(_p(m), _p(g), g_dtype, m.size, beta1, _p(s))
    return s


def zero_rule(s, step, rule=ZERO_ALT):
    s = _arr(s, np.int8)
    b = np.empty(s.shape, np.uint8)
    _zero_rule(_p(s), s.size, step, rule, _p(b))
    return b


def pack_1bit(b):
    b = _arr(b, np.uint8)
    words = np.empty(n_words(b.size), np.uint64)
    _pack_1bit(_p(b), b.size, _p(words))
    return words


def unpack_1bit(words, n):
    words = _arr(words, np.uint64)
    assert words.size >= n_words(n)
    b = np.empty(n, np.uint8)
    _unpack_1bit(_p(words), n, _p(b))
    return b


def container_bits(p):
    return int(_container_bits(p))


def field_bytes(n, p):
    per = 8 // container_bits(p)
    return (n + per - 1) // per


def pack_fields(v, p):
    v = _arr(v, np.uint8)
    if container_bits(p) < 0:
        raise OracleError(ERR_RANGE, "pack_fields")
    out = np.empty(field_bytes(v.size, p), np.uint8)
    rc = _pack_fields(_p(v), v.size, p, _p(out))
    if rc:
        raise OracleError(rc, "pack_fields")
    return out


def unpack_fields(bytes_, n, p):
    bytes_ = _arr(bytes_, np.uint8)
    if container_bits(p) < 0:
        raise OracleError(ERR_RANGE, "unpack_fields")
    assert bytes_.size >= field_bytes(n, p)
    v = np.empty(n, np.uint8)
    rc = _unpack_fields(_p(bytes_), n, p, _p(v))
    if rc:
        raise OracleError(rc, "unpack_fields")
    return v


def count_sign(b, step, tie_rule=TIE_ZERO, p=0):
    """b: (W, n) array of 0/1.  Returns K, S (int32) and u (int8)."""
    b = _arr(b, np.uint8)
    assert b.ndim == 2
    W, n = b.shape
    K = np.empty(n, np.int32)
    S = np.empty(n, np.int32)
    u = np.empty(n, np.int8)
    rc = _count_sign(_p(b), W, n, p, step, tie_rule, _p(K), _p(S), _p(u))
    if rc:
        raise OracleError(rc, "count_sign")
    return K, S, u


def planes(u):
    u = _arr(u, np.int8)
    pos = np.empty(n_words(u.size), np.uint64)
    nz = np.empty(n_words(u.size), np.uint64)
    _planes(_p(u), u.size, _p(pos), _p(nz))
    return pos, nz


def unplanes(pos, nz, n):
    pos = _arr(pos, np.uint64)
    nz = _arr(nz, np.uint64)
    u = np.empty(n, np.int8)
    _unplanes(_p(pos), _p(nz), n, _p(u))
    return u


def apply(theta, u, lr, wd):
    theta = _arr(theta, np.float32)
    u = _arr(u, np.int8)
    assert theta.shape == u.shape
    out = np.empty(theta.shape, np.float64)
    _apply(_p(theta), _p(u), theta.size, lr, wd, _p(out))
    return out


def momentum(m, g, beta2, g_dtype=F32):
    m = _arr(m, np.float32)
    g = _grad(g, g_dtype)
    assert g.shape == m.shape
    out = np.empty(m.shape, np.float64)
    _momentum(_p(m), _p(g), g_dtype, m.size, beta2, _p(out))
    return out


def momentum_avg(m):
    """m: (W, n) float32.  Returns the fp64 mean over W, shape (n,)."""
    m = _arr(m, np.float32)
    assert m.ndim == 2
    W, n = m.shape
    out = np.empty(n, np.float64)
    _momentum_avg(_p(m), W, n, _p(out))
    return out


def sum_bytes(bytes_):
    """bytes_: (W, nbytes) uint8 packed containers.  Byte-wise sum mod 256."""
    bytes_ = _arr(bytes_, np.uint8)
    assert bytes_.ndim == 2
    W, nb = bytes_.shape
    out = np.empty(nb, np.uint8)
    _sum_bytes(_p(bytes_), W, nb, _p(out))
    return out


def _local_bits(m, g, beta1, step, zero, g_dtype):
    W = len(m)
    s = np.stack([local_sign(m[w], g[w], beta1, g_dtype) for w in range(W)])
    b = np.stack([zero_rule(s[w], step, zero) for w in range(W)])
    return s, b


def step_1bit(theta, m, g, *, beta1, beta2, lr, wd, step, zero=ZERO_ALT, tie=TIE_ZERO,
              g_dtype=F32):
    """One whole step on the 1-bit path, in the order of Algorithm 1.

    theta (n,), m (W, n), g (W, n).  Each worker signs its interpolation, forces zeros,
    packs; the W packed buffers are unpacked, summed, signed (the local part of the
    1-bit compressed allreduce of Section 3); the vote is applied to theta and every
    worker updates its own momentum from the momentum it started with.
    """
    m = _arr(m, np.float32)
    W, n = m.shape
    s, b = _local_bits(m, g, beta1, step, zero, g_dtype)
    words = np.stack([pack_1bit(b[w]) for w in range(W)])
    back = np.stack([unpack_1bit(words[w], n) for w in range(W)])
    K, S, u = count_sign(back, step, tie)
    pos, nz = planes(u)
    theta_new = apply(theta, u, lr, wd)
    m_new = np.stack([momentum(m[w], g[w], beta2, g_dtype) for w in range(W)])
    return dict(s=s, b=b, words=words, K=K, S=S, u=u, pos=pos, nz=nz,
                theta=theta_new, m=m_new)


def step_pbit(theta, m, g, *, p, beta1, beta2, lr, wd, step, zero=ZERO_ALT, tie=TIE_ZERO,
              g_dtype=F32):
    """One whole step on the p-bit path (Section 3 "direct allreduce", Appendix F.1).

    Signs go to {0,1} in p-bit fields of uint8 containers; the containers are summed
    as integers; the fields of the sum are the counts K.
    """
    m = _arr(m, np.float32)
    W, n = m.shape
    if p < 1 or p > 8 or W > (1 << p) - 1:
        raise OracleError(ERR_RANGE, "step_pbit")
    s, b = _local_bits(m, g, beta1, step, zero, g_dtype)
    fields = np.stack([pack_fields(b[w], p) for w in range(W)])
    total = sum_bytes(fields)
    K8 = unpack_fields(total, n, p)
    K, S, u = count_sign(b, step, tie, p)
    assert np.array_equal(K, K8.astype(np.int32))
    pos, nz = planes(u)
    theta_new = apply(theta, u, lr, wd)
    m_new = np.stack([momentum(m[w], g[w], beta2, g_dtype) for w in range(W)])
    return dict(s=s, b=b, fields=fields, sum_fields=total, K=K, S=S, u=u, pos=pos, nz=nz,
                theta=theta_new, m=m_new)


# ---- L1 quantisation (Section 4.2, Equation 1 with p = 1) -------------------------------
_local_c = _sig("orc_local_c", None, _vp, _vp, _i, _sz, _f, _vp)
_abs_totals = _sig("orc_abs_totals", None, _vp, _sz, _vp)
_l1_levels = _sig("orc_l1_levels", None, _vp, _sz, C.c_double, _i, _vp)
_level_sum_sign = _sig("orc_level_sum_sign", _i, _vp, _i, _sz, _i, _u64, _i, _vp, _vp, _vp)


def local_c(m, g, beta1, g_dtype=F32):
    """Algorithm 1 line 3: the interpolation itself, float32."""
    m = _arr(m, np.float32)
    g = _grad(g, g_dtype)
    c = np.empty(m.shape, np.float32)
    _local_c(_p(m), _p(g), g_dtype, m.size, beta1, _p(c))
    return c


def mean_abs(x):
    """M_1(x) = (1/d) sum |x_j| of Equation 1: the sum is formed without rounding (integer
    totals per binary exponent, added as Python integers), rounded once to fp64, and
    divided by d in fp64."""
    x = _arr(x, np.float32).ravel()
    totals = np.zeros(256, np.uint64)
    _abs_totals(_p(x), x.size, _p(totals))
    if totals[255]:
        return float("nan")
    exact = sum(int(t) << (e - 1) for e, t in enumerate(totals.tolist()) if t)   # units of 2^-149
    return float(np.ldexp(float(exact), -149)) / x.size if x.size else 0.0


def l1_levels(x, mean, L):
    x = _arr(x, np.float32)
    out = np.empty(x.shape, np.int8)
    _l1_levels(_p(x), x.size, float(mean), L, _p(out))
    return out


def level_sum_sign(rows, L, step, tie_rule=TIE_ZERO):
    """rows: (W, n) uint8 biased levels.  Returns K, S (int32), u (int8)."""
    rows = _arr(rows, np.uint8)
    W, n = rows.shape
    K = np.empty(n, np.int32)
    S = np.empty(n, np.int32)
    u = np.empty(n, np.int8)
    rc = _level_sum_sign(_p(rows), W, n, L, step, tie_rule, _p(K), _p(S), _p(u))
    if rc:
        raise OracleError(rc, "level_sum_sign")
    return K, S, u


def step_l1(theta, m, g, *, L, beta1, beta2, lr, wd, step, tie=TIE_ZERO, g_dtype=F32):
    """One whole step with L1-quantised updates (Equation 1, Appendix F.1): every worker
    scales its interpolation by L / (2 mean|c|), rounds, clamps to [-L, L] and sends
    level + L as a byte; the bytes are summed, the sign of the summed levels moves theta."""
    m = _arr(m, np.float32)
    W, n = m.shape
    if 2 * L * W > 255:
        raise OracleError(ERR_RANGE, "step_l1")
    c = np.stack([local_c(m[w], g[w], beta1, g_dtype) for w in range(W)])
    means = np.array([mean_abs(c[w]) for w in range(W)])
    levels = np.stack([l1_levels(c[w], means[w], L) for w in range(W)])
    fields = (levels.astype(np.int16) + L).astype(np.uint8)
    K, S, u = level_sum_sign(fields, L, step, tie)
    assert np.array_equal(sum_bytes(fields), K.astype(np.uint8))
    pos, nz = planes(u)
    theta_new = apply(theta, u, lr, wd)
    m_new = np.stack([momentum(m[w], g[w], beta2, g_dtype) for w in range(W)])
    return dict(c=c, mean_abs=means, levels=levels, fields=fields, K=K, S=S, u=u, pos=pos, nz=nz,
                theta=theta_new, m=m_new)


# ---- ternary wire format (Appendix B.1) --------------------------------------------------
_ternary_vote = _sig("orc_ternary_vote", _i, _vp, _i, _sz, _vp, _vp, _vp, _vp)


def ternary_vote(s):
    """s: (W, n) int8 signs in {-1, 0, +1}.  Returns Kp, Kn, S (int32) and u (int8)."""
    s = _arr(s, np.int8)
    W, n = s.shape
    Kp, Kn, S = (np.empty(n, np.int32) for _ in range(3))
    u = np.empty(n, np.int8)
    rc = _ternary_vote(_p(s), W, n, _p(Kp), _p(Kn), _p(S), _p(u))
    if rc:
        raise OracleError(rc, "ternary_vote")
    return Kp, Kn, S, u


def step_ternary(theta, m, g, *, beta1, beta2, lr, wd, g_dtype=F32):
    """One whole step with exact zeros on the wire: each worker's ternary sign travels as
    two 1-bit planes (pos = s > 0, nz = s != 0); the update is sign(sum of signs)."""
    m = _arr(m, np.float32)
    W, n = m.shape
    s = np.stack([local_sign(m[w], g[w], beta1, g_dtype) for w in range(W)])
    pl = [planes(s[w]) for w in range(W)]
    pos_w = np.stack([p[0] for p in pl])
    nz_w = np.stack([p[1] for p in pl])
    back = np.stack([unplanes(pos_w[w], nz_w[w], n) for w in range(W)])
    Kp, Kn, S, u = ternary_vote(back)
    pos, nz = planes(u)
    theta_new = apply(theta, u, lr, wd)
    m_new = np.stack([momentum(m[w], g[w], beta2, g_dtype) for w in range(W)])
    return dict(s=s, pos_w=pos_w, nz_w=nz_w, Kp=Kp, Kn=Kn, S=S, u=u, pos=pos, nz=nz, theta=theta_new, m=m_new)


# ---- divergence of the workers' momenta (Section 5.1) ------------------------------------
_momentum_divergence = _sig("orc_momentum_divergence", C.c_double, _vp, _i, _sz)


def momentum_divergence(m):
    """m: (W, n) float32.  max over elements of the standard deviation across workers."""
    m = _arr(m, np.float32)
    W, n = m.shape
    return float(_momentum_divergence(_p(m), W, n))
