"""The C-ABI library loads, exports every symbol include/lioncub.h declares, and its
host-side validation returns the documented status codes before anything is launched.
No GPU needed: no call here reaches a kernel launch."""
import ctypes
import os
import re

import pytest

import paper_2411_16462_amd as lc
from conftest import ROOT

HEADER = os.path.join(ROOT, "include", "lioncub.h")
A = 0x7F0000001000  # a 4 KiB-aligned address that is never dereferenced on the host


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lc_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported_and_bound():
    names = declared_functions()
    assert {"lc_local_update_pack", "lc_vote_1bit", "lc_pbit_sum_sign", "lc_apply_update",
            "lc_momentum_avg"} <= set(names)
    raw = ctypes.CDLL(lc.LIB_PATH)
    for name in names:
        assert hasattr(raw, name), "library does not export " + name
        assert name in lc.SIGNATURES, "binding does not cover " + name
        assert callable(getattr(lc, name))
    assert set(lc.SIGNATURES) == set(names)


def test_binding_constants_match_header():
    text = open(HEADER).read()
    for name in ("LC_OK", "LC_ERR_NULL", "LC_ERR_SIZE", "LC_ERR_ALIGN", "LC_ERR_RANGE", "LC_ERR_DTYPE",
                 "LC_ERR_MODE", "LC_F32", "LC_BF16", "LC_ZERO_ALT", "LC_ZERO_POS", "LC_ZERO_NEG",
                 "LC_TIE_ZERO", "LC_TIE_ALT"):
        m = re.search(r"\b%s\s*=\s*(\d+)" % name, text)
        assert m and int(m.group(1)) == getattr(lc, name), name
    assert int(re.search(r"#define LC_MAX_W (\d+)", text).group(1)) == lc.LC_MAX_W
    assert int(re.search(r"#define LC_L1_WORKSPACE_WORDS (\d+)", text).group(1)) == lc.LC_L1_WORKSPACE_WORDS


def test_version_status_strings_and_container_rule():
    assert lc.lc_version() >= 100
    for code in range(0, 7):
        assert lc.lc_status_string(code).startswith("LC_")
    assert "HIP" in lc.lc_status_string(-1)
    assert [lc.lc_container_bits(p) for p in range(0, 10)] == [-1, 1, 2, 4, 4, 8, 8, 8, 8, -1]


def pack(**kw):
    a = dict(g=A, g_stride_elems=1024, g_dtype=lc.LC_F32, m=A, m_stride_elems=1024, W=4, n=1000, beta1=0.9,
             update_m=1, beta2=0.99, out_bits=1, q=A, q_stride_bytes=128, step=1, zero_rule=lc.LC_ZERO_ALT,
             stream=0, check=False)
    a.update(kw)
    return lc.lc_local_update_pack(**a)


def test_update_pack_validation():
    assert pack(n=0) == lc.LC_OK                               # empty range: successful no-op
    assert pack(W=0) == lc.LC_ERR_SIZE
    assert pack(W=lc.LC_MAX_W + 1) == lc.LC_ERR_SIZE
    assert pack(g=None) == lc.LC_ERR_NULL
    assert pack(m=None) == lc.LC_ERR_NULL
    assert pack(q=None, update_m=0) == lc.LC_ERR_NULL
    assert pack(q=None, update_m=1, n=0) == lc.LC_OK
    assert pack(g_dtype=2) == lc.LC_ERR_DTYPE
    assert pack(out_bits=3) == lc.LC_ERR_MODE
    assert pack(out_bits=16) == lc.LC_ERR_MODE
    assert pack(zero_rule=3) == lc.LC_ERR_MODE
    assert pack(m=A + 4) == lc.LC_ERR_ALIGN
    assert pack(g=A + 8) == lc.LC_ERR_ALIGN
    assert pack(m_stride_elems=1001) == lc.LC_ERR_ALIGN
    assert pack(g_stride_elems=1004, g_dtype=lc.LC_BF16) == lc.LC_ERR_ALIGN   # 2008 bytes
    assert pack(g_stride_elems=1001, W=1, n=0) == lc.LC_OK                     # one row: stride unused
    assert pack(q=A + 4) == lc.LC_ERR_ALIGN
    assert pack(q_stride_bytes=12) == lc.LC_ERR_ALIGN
    assert pack(out_bits=4, q=A + 8) == lc.LC_ERR_ALIGN                        # field rows: 16 bytes
    with pytest.raises(lc.LionCubError) as e:
        pack(W=0, check=True)
    assert e.value.status == lc.LC_ERR_SIZE


def test_vote_and_sum_validation():
    v = dict(q=A, q_stride_words=16, W=4, n=0, vote_pos=A, vote_nz=A, step=1, tie_rule=lc.LC_TIE_ZERO,
             stream=0, check=False)
    assert lc.lc_vote_1bit(**v) == lc.LC_OK
    assert lc.lc_vote_1bit(**{**v, "W": 256}) == lc.LC_ERR_SIZE
    assert lc.lc_vote_1bit(**{**v, "q": None}) == lc.LC_ERR_NULL
    assert lc.lc_vote_1bit(**{**v, "tie_rule": 2}) == lc.LC_ERR_MODE
    assert lc.lc_vote_1bit(**{**v, "q": A + 4}) == lc.LC_ERR_ALIGN
    assert lc.lc_vote_1bit(**{**v, "vote_pos": A + 4}) == lc.LC_ERR_ALIGN
    s = dict(q=A, q_stride_bytes=512, in_bits=4, W=8, n=0, p=4, sum_out=A, vote_pos=None, vote_nz=None,
             step=1, tie_rule=lc.LC_TIE_ZERO, stream=0, check=False)
    assert lc.lc_pbit_sum_sign(**s) == lc.LC_OK
    # range rule of the p-bit sum: W <= 2^p - 1 (four bits cannot serve sixteen workers)
    assert lc.lc_pbit_sum_sign(**{**s, "W": 15}) == lc.LC_OK
    assert lc.lc_pbit_sum_sign(**{**s, "W": 16}) == lc.LC_ERR_RANGE
    assert lc.lc_pbit_sum_sign(**{**s, "p": 3, "W": 7}) == lc.LC_OK         # 3 bits live in a nibble
    assert lc.lc_pbit_sum_sign(**{**s, "p": 3, "W": 8}) == lc.LC_ERR_RANGE
    assert lc.lc_pbit_sum_sign(**{**s, "p": 7, "in_bits": 1, "W": 64}) == lc.LC_OK
    assert lc.lc_pbit_sum_sign(**{**s, "p": 6, "in_bits": 1, "W": 64}) == lc.LC_ERR_RANGE
    assert lc.lc_pbit_sum_sign(**{**s, "p": 8, "in_bits": 8, "W": 125}) == lc.LC_OK
    assert lc.lc_pbit_sum_sign(**{**s, "p": 0}) == lc.LC_ERR_RANGE
    assert lc.lc_pbit_sum_sign(**{**s, "p": 9}) == lc.LC_ERR_RANGE
    assert lc.lc_pbit_sum_sign(**{**s, "in_bits": 2}) == lc.LC_ERR_MODE       # must be 1 or container(p)
    assert lc.lc_pbit_sum_sign(**{**s, "q": A + 8}) == lc.LC_ERR_ALIGN
    assert lc.lc_pbit_sum_sign(**{**s, "q_stride_bytes": 520}) == lc.LC_ERR_ALIGN
    assert lc.lc_pbit_sum_sign(**{**s, "sum_out": A + 8}) == lc.LC_ERR_ALIGN


def test_apply_avg_and_fused_validation():
    a = dict(theta=A, vote_pos=A, vote_nz=A, n=0, lr=1e-4, wd=0.1, m=None, m_stride_elems=0, g=None,
             g_stride_elems=0, g_dtype=lc.LC_F32, n_m=0, beta2=0.99, stream=0, check=False)
    assert lc.lc_apply_update(**a) == lc.LC_OK
    assert lc.lc_apply_update(**{**a, "vote_nz": None}) == lc.LC_OK           # one-plane update
    assert lc.lc_apply_update(**{**a, "theta": None}) == lc.LC_ERR_NULL
    assert lc.lc_apply_update(**{**a, "vote_pos": None}) == lc.LC_ERR_NULL
    assert lc.lc_apply_update(**{**a, "theta": A + 4}) == lc.LC_ERR_ALIGN
    assert lc.lc_apply_update(**{**a, "n_m": 1}) == lc.LC_ERR_NULL            # needs m and g
    assert lc.lc_apply_update(**{**a, "n_m": -1}) == lc.LC_ERR_SIZE
    assert lc.lc_apply_update(**{**a, "n_m": 1, "m": A, "g": A, "g_dtype": 7}) == lc.LC_ERR_DTYPE
    assert lc.lc_momentum_avg(A, 1024, 4, 0, stream=0, check=False) == lc.LC_OK
    assert lc.lc_momentum_avg(None, 1024, 4, 10, stream=0, check=False) == lc.LC_ERR_NULL
    assert lc.lc_momentum_avg(A, 1023, 4, 10, stream=0, check=False) == lc.LC_ERR_ALIGN
    assert lc.lc_momentum_avg(A, 1024, 0, 10, stream=0, check=False) == lc.LC_ERR_SIZE
    assert lc.lc_momentum_avg(A, 1023, 1, 10, stream=0, check=False) == lc.LC_OK   # W = 1: nothing to do
    f = dict(q=A, q_stride_words=16, W=4, n=0, step=1, tie_rule=lc.LC_TIE_ZERO, theta=A, lr=1e-4, wd=0.1,
             m=None, m_stride_elems=0, g=None, g_stride_elems=0, g_dtype=lc.LC_F32, n_m=0, beta2=0.99,
             stream=0, check=False)
    assert lc.lc_vote_apply_1bit(**f) == lc.LC_OK
    assert lc.lc_vote_apply_1bit(**{**f, "theta": None}) == lc.LC_ERR_NULL
    assert lc.lc_vote_apply_1bit(**{**f, "n_m": 2}) == lc.LC_ERR_NULL
    pa = dict(q=A, q_stride_bytes=512, in_bits=4, W=8, n=0, p=4, sum_out=None, step=1,
              tie_rule=lc.LC_TIE_ZERO, theta=A, lr=1e-4, wd=0.1, m=None, m_stride_elems=0, g=None,
              g_stride_elems=0, g_dtype=lc.LC_F32, n_m=0, beta2=0.99, stream=0, check=False)
    assert lc.lc_pbit_sum_apply(**pa) == lc.LC_OK
    assert lc.lc_pbit_sum_apply(**{**pa, "W": 16}) == lc.LC_ERR_RANGE
    assert lc.lc_pbit_sum_apply(**{**pa, "theta": None}) == lc.LC_ERR_NULL


def test_l1_validation():
    mean = dict(g=A, g_stride_elems=1024, g_dtype=lc.LC_F32, m=A, m_stride_elems=1024, W=4, n=0, beta1=0.9, mean_abs=A,
                workspace=A, stream=0, check=False)
    assert lc.lc_l1_mean_abs(**{**mean, "W": 0}) == lc.LC_ERR_SIZE
    assert lc.lc_l1_mean_abs(**{**mean, "mean_abs": None}) == lc.LC_ERR_NULL
    assert lc.lc_l1_mean_abs(**{**mean, "workspace": None}) == lc.LC_ERR_NULL
    assert lc.lc_l1_mean_abs(**{**mean, "workspace": A + 4}) == lc.LC_ERR_ALIGN
    assert lc.lc_l1_mean_abs(**{**mean, "g_dtype": 3}) == lc.LC_ERR_DTYPE
    qz = dict(g=A, g_stride_elems=1024, g_dtype=lc.LC_F32, m=A, m_stride_elems=1024, W=4, n=0, beta1=0.9, update_m=1,
              beta2=0.99, levels=15, mean_abs=A, q=A, q_stride_bytes=1024, stream=0, check=False)
    assert lc.lc_l1_quantize_pack(**qz) == lc.LC_OK
    assert lc.lc_l1_quantize_pack(**{**qz, "levels": 0}) == lc.LC_ERR_RANGE
    assert lc.lc_l1_quantize_pack(**{**qz, "levels": 128}) == lc.LC_ERR_RANGE
    assert lc.lc_l1_quantize_pack(**{**qz, "q": None}) == lc.LC_ERR_NULL
    assert lc.lc_l1_quantize_pack(**{**qz, "q_stride_bytes": 1000}) == lc.LC_ERR_ALIGN
    sm = dict(q=A, q_stride_bytes=1024, W=8, n=0, levels=15, sum_out=A, vote_pos=A, vote_nz=A, step=1,
              tie_rule=lc.LC_TIE_ZERO, stream=0, check=False)
    assert lc.lc_level_sum_sign(**sm) == lc.LC_OK                       # 8 workers x 30 = 240 fits a byte
    assert lc.lc_level_sum_sign(**{**sm, "W": 9}) == lc.LC_ERR_RANGE    # 270 does not
    assert lc.lc_level_sum_sign(**{**sm, "levels": 127, "W": 1}) == lc.LC_OK
    assert lc.lc_level_sum_sign(**{**sm, "levels": 127, "W": 2}) == lc.LC_ERR_RANGE
    assert lc.lc_level_sum_sign(**{**sm, "levels": 0}) == lc.LC_ERR_RANGE
    ap = dict(q=A, q_stride_bytes=1024, W=8, n=0, levels=15, sum_out=None, step=1, tie_rule=lc.LC_TIE_ZERO, theta=A,
              lr=1e-4, wd=0.1, m=None, m_stride_elems=0, g=None, g_stride_elems=0, g_dtype=lc.LC_F32, n_m=0, beta2=0.99,
              stream=0, check=False)
    assert lc.lc_level_sum_apply(**ap) == lc.LC_OK
    assert lc.lc_level_sum_apply(**{**ap, "theta": None}) == lc.LC_ERR_NULL
    assert lc.lc_level_sum_apply(**{**ap, "W": 9}) == lc.LC_ERR_RANGE


def test_ternary_validation():
    pk = dict(g=A, g_stride_elems=1024, g_dtype=lc.LC_F32, m=A, m_stride_elems=1024, W=4, n=0, beta1=0.9, update_m=1,
              beta2=0.99, pos=A, nz=A, q_stride_words=16, stream=0, check=False)
    assert lc.lc_local_update_pack_ternary(**pk) == lc.LC_OK
    assert lc.lc_local_update_pack_ternary(**{**pk, "nz": None}) == lc.LC_ERR_NULL
    assert lc.lc_local_update_pack_ternary(**{**pk, "pos": A + 4}) == lc.LC_ERR_ALIGN
    assert lc.lc_local_update_pack_ternary(**{**pk, "W": 256}) == lc.LC_ERR_SIZE
    vt = dict(pos=A, nz=A, q_stride_words=16, W=4, n=0, vote_pos=A, vote_nz=None, stream=0, check=False)
    assert lc.lc_vote_ternary(**vt) == lc.LC_OK
    assert lc.lc_vote_ternary(**{**vt, "nz": None}) == lc.LC_ERR_NULL
    assert lc.lc_vote_ternary(**{**vt, "nz": A + 4}) == lc.LC_ERR_ALIGN
    va = dict(pos=A, nz=A, q_stride_words=16, W=4, n=0, theta=A, lr=1e-4, wd=0.1, m=None, m_stride_elems=0, g=None,
              g_stride_elems=0, g_dtype=lc.LC_F32, n_m=0, beta2=0.99, stream=0, check=False)
    assert lc.lc_vote_apply_ternary(**va) == lc.LC_OK
    assert lc.lc_vote_apply_ternary(**{**va, "theta": None}) == lc.LC_ERR_NULL
    assert lc.lc_vote_apply_ternary(**{**va, "n_m": 1}) == lc.LC_ERR_NULL


def test_divergence_and_sync_ranges_validation():
    d = dict(m=A, m_stride_elems=1024, W=4, n=0, max_std=A, stream=0, check=False)
    assert lc.lc_momentum_divergence(**{**d, "m": None}) == lc.LC_ERR_NULL
    assert lc.lc_momentum_divergence(**{**d, "max_std": None}) == lc.LC_ERR_NULL
    assert lc.lc_momentum_divergence(**{**d, "max_std": A + 4}) == lc.LC_ERR_ALIGN
    assert lc.lc_momentum_divergence(**{**d, "W": 0}) == lc.LC_ERR_SIZE
    s = dict(m=A, m_stride_elems=1024, W=4, offsets=[0, 64], sizes=[64, 128], n_ranges=2, step=3, every=10, stream=0,
             check=False)
    assert lc.lc_momentum_sync_ranges(**s) == lc.LC_OK                      # step 3 of every 10: nothing to do
    assert lc.lc_momentum_sync_ranges(**{**s, "every": 0}) == lc.LC_ERR_MODE
    assert lc.lc_momentum_sync_ranges(**{**s, "offsets": [0, 66]}) == lc.LC_ERR_ALIGN
    assert lc.lc_momentum_sync_ranges(**{**s, "offsets": None}) == lc.LC_ERR_NULL
    assert lc.lc_momentum_sync_ranges(**{**s, "m": None}) == lc.LC_ERR_NULL
    assert lc.lc_momentum_sync_ranges(**{**s, "n_ranges": 0, "step": 10}) == lc.LC_OK
    assert lc.lc_momentum_sync_ranges(**{**s, "sizes": [0, 0], "step": 10}) == lc.LC_OK   # empty ranges: no launch


def test_element_and_group_count_limits():
    """n beyond LC_MAX_N and group counts outside 1..LC_MAX_GROUPS are refused before any
    launch, by every entry point that takes them."""
    text = open(HEADER).read()
    assert "#define LC_MAX_N ((size_t)1 << 38)" in text and lc.LC_MAX_N == 1 << 38
    assert "#define LC_MAX_GROUPS (1 << 20)" in text and lc.LC_MAX_GROUPS == 1 << 20
    big = lc.LC_MAX_N + 1
    assert pack(n=big) == lc.LC_ERR_SIZE
    assert lc.lc_vote_1bit(A, 16, 4, big, A, A, 1, lc.LC_TIE_ZERO, stream=0, check=False) == lc.LC_ERR_SIZE
    assert lc.lc_pbit_sum_sign(A, 512, 4, 8, big, 4, A, None, None, 1, lc.LC_TIE_ZERO, stream=0, check=False) == lc.LC_ERR_SIZE
    assert lc.lc_apply_update(A, A, A, big, 1e-4, 0.1, None, 0, None, 0, lc.LC_F32, 0, 0.99, stream=0,
                              check=False) == lc.LC_ERR_SIZE
    assert lc.lc_momentum_avg(A, 1024, 4, big, stream=0, check=False) == lc.LC_ERR_SIZE
    assert lc.lc_momentum_divergence(A, 1024, 4, big, A, stream=0, check=False) == lc.LC_ERR_SIZE
    assert lc.lc_l1_mean_abs(A, 1024, lc.LC_F32, A, 1024, 4, big, 0.9, A, A, stream=0, check=False) == lc.LC_ERR_SIZE
    assert lc.lc_l1_quantize_pack(A, 1024, lc.LC_F32, A, 1024, 4, big, 0.9, 1, 0.99, 15, A, A, 1024, stream=0,
                                  check=False) == lc.LC_ERR_SIZE
    assert lc.lc_local_update_pack_ternary(A, 1024, lc.LC_F32, A, 1024, 4, big, 0.9, 1, 0.99, A, A, 16, stream=0,
                                           check=False) == lc.LC_ERR_SIZE
    for G in (0, -3, lc.LC_MAX_GROUPS + 1):
        assert lc.lc_vote_apply_1bit_groups(A, 16, 4, 0, 1, lc.LC_TIE_ZERO, A, A, A, A, G, stream=0,
                                            check=False) == lc.LC_ERR_SIZE
        assert lc.lc_pbit_sum_apply_groups(A, 512, 4, 8, 0, 4, None, 1, lc.LC_TIE_ZERO, A, A, A, A, G, stream=0,
                                           check=False) == lc.LC_ERR_SIZE
        assert lc.lc_vote_apply_ternary_groups(A, A, 16, 4, 0, A, A, A, A, G, stream=0, check=False) == lc.LC_ERR_SIZE
        assert lc.lc_level_sum_apply_groups(A, 1024, 4, 0, 15, None, 1, lc.LC_TIE_ZERO, A, A, A, A, G, stream=0,
                                            check=False) == lc.LC_ERR_SIZE
        assert lc.lc_l1_mean_abs_groups(A, 1024, lc.LC_F32, A, 1024, 4, 0, 0.9, A, None, G, A, A, stream=0,
                                        check=False) == lc.LC_ERR_SIZE
        assert lc.lc_l1_quantize_pack_groups(A, 1024, lc.LC_F32, A, 1024, 4, 0, 0.9, 1, 0.99, 15, A, G, A, A, 1024,
                                             stream=0, check=False) == lc.LC_ERR_SIZE
    # a valid table with n = 0 is a no-op
    assert lc.lc_vote_apply_1bit_groups(A, 16, 4, 0, 1, lc.LC_TIE_ZERO, A, A, A, A, 3, stream=0, check=False) == lc.LC_OK
    assert lc.lc_l1_quantize_pack_groups(A, 1024, lc.LC_F32, A, 1024, 4, 0, 0.9, 1, 0.99, 15, A, 3, A, A, 1024, stream=0,
                                         check=False) == lc.LC_OK
    assert lc.lc_l1_groups_workspace_words(8, 148) == 8 * 148 * lc.LC_L1_WORKSPACE_WORDS + 75


def test_count_apply_validation():
    a = dict(k_fields=A, field_bits=4, n=0, total=8, step=1, tie_rule=lc.LC_TIE_ZERO, theta=A, lr=1e-4, wd=0.1, m=None,
             m_stride_elems=0, g=None, g_stride_elems=0, g_dtype=lc.LC_F32, n_m=0, beta2=0.99, stream=0, check=False)
    assert lc.lc_count_apply(**a) == lc.LC_OK
    assert lc.lc_count_apply(**{**a, "total": 15}) == lc.LC_OK
    assert lc.lc_count_apply(**{**a, "total": 16}) == lc.LC_ERR_RANGE          # a nibble cannot hold 16
    assert lc.lc_count_apply(**{**a, "total": 0}) == lc.LC_ERR_RANGE
    assert lc.lc_count_apply(**{**a, "field_bits": 8, "total": 255}) == lc.LC_OK
    assert lc.lc_count_apply(**{**a, "field_bits": 8, "total": 256}) == lc.LC_ERR_RANGE
    assert lc.lc_count_apply(**{**a, "field_bits": 2, "total": 3}) == lc.LC_OK
    assert lc.lc_count_apply(**{**a, "field_bits": 1, "total": 1}) == lc.LC_ERR_MODE
    assert lc.lc_count_apply(**{**a, "field_bits": 3}) == lc.LC_ERR_MODE
    assert lc.lc_count_apply(**{**a, "tie_rule": 2}) == lc.LC_ERR_MODE
    assert lc.lc_count_apply(**{**a, "k_fields": None}) == lc.LC_ERR_NULL
    assert lc.lc_count_apply(**{**a, "theta": None}) == lc.LC_ERR_NULL
    assert lc.lc_count_apply(**{**a, "k_fields": A + 8}) == lc.LC_ERR_ALIGN
    assert lc.lc_count_apply(**{**a, "n_m": 1}) == lc.LC_ERR_NULL             # momentum rows need m and g
    assert lc.lc_count_apply(**{**a, "n": lc.LC_MAX_N + 1}) == lc.LC_ERR_SIZE


def test_group_table_limits_and_signatures():
    """*_groups calls: the element count must fit the 32-bit segment ends (64 * (2^32 - 1)),
    and no grouped apply takes momentum rows -- its signature has no m / g / n_m at all, so
    such a call cannot be expressed."""
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    grouped = re.findall(r"int (lc_\w+_groups)\s*\(([^;]*?)\);", text, flags=re.S)
    assert len(grouped) >= 7
    for name, params in grouped:
        if "_apply_" in name:
            assert not re.search(r"\bn_m\b|\*\s*m\b|\*\s*g\b|beta2", params), name
    too_long = 64 * (2 ** 32 - 1) + 64
    assert too_long <= lc.LC_MAX_N
    v = dict(q=A, q_stride_words=1 << 33, W=4, n=too_long, step=1, tie_rule=lc.LC_TIE_ZERO, theta=A, group_end64=A,
             group_lr=A, group_wd=A, n_groups=3, stream=0, check=False)
    assert lc.lc_vote_apply_1bit_groups(**v) == lc.LC_ERR_SIZE
    assert lc.lc_vote_apply_1bit_groups(**{**v, "n": 0}) == lc.LC_OK
    assert lc.lc_vote_apply_1bit_groups(**{**v, "n": 0, "n_groups": 0}) == lc.LC_ERR_SIZE
    assert lc.lc_vote_apply_1bit_groups(**{**v, "n": 0, "n_groups": lc.LC_MAX_GROUPS + 1}) == lc.LC_ERR_SIZE
    assert lc.lc_vote_apply_1bit_groups(**{**v, "n": 0, "group_lr": None}) == lc.LC_ERR_NULL
    assert lc.lc_vote_apply_1bit_groups(**{**v, "n": 0, "group_end64": A + 2}) == lc.LC_ERR_ALIGN
    d = dict(m=A, m_stride_elems=1 << 40, W=2, n=too_long, group_end64=A, n_groups=3, max_std=A, stream=0, check=False)
    assert lc.lc_momentum_divergence_groups(**d) == lc.LC_ERR_SIZE
    g = dict(g=A, g_stride_elems=1 << 40, g_dtype=lc.LC_F32, m=A, m_stride_elems=1 << 40, W=2, n=too_long, beta1=0.9,
             group_end64=A, group_count=None, n_groups=3, mean_abs=A, workspace=A, stream=0, check=False)
    assert lc.lc_l1_mean_abs_groups(**g) == lc.LC_ERR_SIZE
    qz = dict(g=A, g_stride_elems=1 << 40, g_dtype=lc.LC_F32, m=A, m_stride_elems=1 << 40, W=2, n=too_long, beta1=0.9,
              update_m=1, beta2=0.99, levels=15, group_end64=A, n_groups=3, mean_abs=A, q=A, q_stride_bytes=1 << 40,
              stream=0, check=False)
    assert lc.lc_l1_quantize_pack_groups(**qz) == lc.LC_ERR_SIZE


def test_static_workspace_entry_point_validation():
    a = dict(g=A, g_stride_elems=1024, g_dtype=lc.LC_F32, m=A, m_stride_elems=1024, n=10, beta1=0.9, mean_abs=A,
             stream=0, check=False)
    assert lc.lc_l1_mean_abs_static(W=lc.LC_L1_STATIC_MAX_W + 1, **a) == lc.LC_ERR_SIZE
    assert lc.lc_l1_mean_abs_static(W=0, **a) == lc.LC_ERR_SIZE
    assert lc.lc_l1_mean_abs_static(W=2, **{**a, "mean_abs": None}) == lc.LC_ERR_NULL
    assert lc.lc_l1_mean_abs_static(W=2, **{**a, "g_dtype": 7}) == lc.LC_ERR_DTYPE
    text = open(HEADER).read()
    assert int(re.search(r"#define LC_L1_STATIC_MAX_W (\d+)", text).group(1)) == lc.LC_L1_STATIC_MAX_W


def test_stream_probe_validation():
    probe = lambda **kw: lc.lc_stream_probe(**dict(dict(kind=lc.LC_PROBE_COPY, a=A, b=A + 4096, n=1000, s=1.0, stream=0, check=False), **kw))
    text = open(HEADER).read()
    for name in ("LC_PROBE_READ", "LC_PROBE_WRITE", "LC_PROBE_COPY", "LC_PROBE_SCALE", "LC_PROBE_RMW2"):
        assert int(re.search(r"#define %s (\d+)" % name, text).group(1)) == getattr(lc, name)
    assert probe(n=0) == lc.LC_OK
    assert probe(kind=-1) == lc.LC_ERR_MODE and probe(kind=5) == lc.LC_ERR_MODE
    assert probe(a=0) == lc.LC_ERR_NULL
    assert probe(b=0) == lc.LC_ERR_NULL and probe(kind=lc.LC_PROBE_RMW2, b=0) == lc.LC_ERR_NULL
    assert probe(kind=lc.LC_PROBE_READ, b=0, n=0) == lc.LC_OK          # b is optional where it is not read
    assert probe(a=A + 4) == lc.LC_ERR_ALIGN and probe(b=A + 8) == lc.LC_ERR_ALIGN
    assert probe(n=lc.LC_MAX_N + 1) == lc.LC_ERR_SIZE
