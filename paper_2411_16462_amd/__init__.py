"""Python binding of liblioncub.so (include/lioncub.h): argument marshalling only.

Every function has the name and the argument order of its C entry point.  Pointer
arguments take a torch tensor on the GPU (its ``data_ptr()`` is passed), ``None`` (NULL)
or an integer device address.  ``stream=None`` means torch's current stream.  A non-zero
status raises ``LionCubError`` unless ``check=False`` is given, in which case the status
is returned.

PyTorch is used for device memory and streams only; every step of the path runs in the
library's kernels.  There is no fallback: if the library has not been built
(``python paper_2411_16462_amd/build.py``) the first call raises.
"""
import ctypes as C
import os

LC_OK, LC_ERR_NULL, LC_ERR_SIZE, LC_ERR_ALIGN, LC_ERR_RANGE, LC_ERR_DTYPE, LC_ERR_MODE = range(7)
LC_F32, LC_BF16 = 0, 1
LC_ZERO_ALT, LC_ZERO_POS, LC_ZERO_NEG = 0, 1, 2
LC_TIE_ZERO, LC_TIE_ALT = 0, 1
LC_PROBE_READ, LC_PROBE_WRITE, LC_PROBE_COPY, LC_PROBE_SCALE, LC_PROBE_RMW2 = 0, 1, 2, 3, 4
LC_MAX_W = 255
LC_L1_WORKSPACE_WORDS = 384
LC_L1_STATIC_MAX_W = 64
LC_MAX_GROUPS = 1 << 20
LC_MAX_N = 1 << 38

# the in-tree build; LIONCUB_LIBRARY names another build of the same library (say one compiled
# with different tuning macros) -- still the HIP library, there is no other implementation
LIB_PATH = os.environ.get("LIONCUB_LIBRARY") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "liblioncub.so")

_vp, _sz, _i, _u64, _f = C.c_void_p, C.c_size_t, C.c_int, C.c_uint64, C.c_float

# name -> (restype, argtypes); mirrors include/lioncub.h
SIGNATURES = {
    "lc_local_update_pack": (_i, [_vp, _sz, _i, _vp, _sz, _i, _sz, _f, _i, _f, _i, _vp, _sz, _u64, _i, _vp]),
    "lc_vote_1bit": (_i, [_vp, _sz, _i, _sz, _vp, _vp, _u64, _i, _vp]),
    "lc_pbit_sum_sign": (_i, [_vp, _sz, _i, _i, _sz, _i, _vp, _vp, _vp, _u64, _i, _vp]),
    "lc_apply_update": (_i, [_vp, _vp, _vp, _sz, _f, _f, _vp, _sz, _vp, _sz, _i, _i, _f, _vp]),
    "lc_count_apply": (_i, [_vp, _i, _sz, _i, _u64, _i, _vp, _f, _f, _vp, _sz, _vp, _sz, _i, _i, _f, _vp]),
    "lc_momentum_avg": (_i, [_vp, _sz, _i, _sz, _vp]),
    "lc_momentum_divergence": (_i, [_vp, _sz, _i, _sz, _vp, _vp]),
    "lc_momentum_divergence_groups": (_i, [_vp, _sz, _i, _sz, _vp, _i, _vp, _vp]),
    "lc_momentum_sync_ranges": (_i, [_vp, _sz, _i, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t), _i, _u64, _u64, _vp]),
    "lc_vote_apply_1bit": (_i, [_vp, _sz, _i, _sz, _u64, _i, _vp, _f, _f, _vp, _sz, _vp, _sz, _i, _i, _f, _vp]),
    "lc_vote_apply_1bit_groups": (_i, [_vp, _sz, _i, _sz, _u64, _i, _vp, _vp, _vp, _vp, _i, _vp]),
    "lc_pbit_sum_apply": (_i, [_vp, _sz, _i, _i, _sz, _i, _vp, _u64, _i, _vp, _f, _f, _vp, _sz, _vp, _sz, _i, _i,
                               _f, _vp]),
    "lc_pbit_sum_apply_groups": (_i, [_vp, _sz, _i, _i, _sz, _i, _vp, _u64, _i, _vp, _vp, _vp, _vp, _i, _vp]),
    "lc_vote_apply_ternary_groups": (_i, [_vp, _vp, _sz, _i, _sz, _vp, _vp, _vp, _vp, _i, _vp]),
    "lc_local_update_pack_ternary": (_i, [_vp, _sz, _i, _vp, _sz, _i, _sz, _f, _i, _f, _vp, _vp, _sz, _vp]),
    "lc_vote_ternary": (_i, [_vp, _vp, _sz, _i, _sz, _vp, _vp, _vp]),
    "lc_vote_apply_ternary": (_i, [_vp, _vp, _sz, _i, _sz, _vp, _f, _f, _vp, _sz, _vp, _sz, _i, _i, _f, _vp]),
    "lc_l1_mean_abs": (_i, [_vp, _sz, _i, _vp, _sz, _i, _sz, _f, _vp, _vp, _vp]),
    "lc_l1_mean_abs_static": (_i, [_vp, _sz, _i, _vp, _sz, _i, _sz, _f, _vp, _vp]),
    "lc_l1_quantize_pack": (_i, [_vp, _sz, _i, _vp, _sz, _i, _sz, _f, _i, _f, _i, _vp, _vp, _sz, _vp]),
    "lc_l1_groups_workspace_words": (_sz, [_i, _i]),
    "lc_l1_mean_abs_groups": (_i, [_vp, _sz, _i, _vp, _sz, _i, _sz, _f, _vp, _vp, _i, _vp, _vp, _vp]),
    "lc_l1_quantize_pack_groups": (_i, [_vp, _sz, _i, _vp, _sz, _i, _sz, _f, _i, _f, _i, _vp, _i, _vp, _vp, _sz, _vp]),
    "lc_level_sum_apply_groups": (_i, [_vp, _sz, _i, _sz, _i, _vp, _u64, _i, _vp, _vp, _vp, _vp, _i, _vp]),
    "lc_level_sum_sign": (_i, [_vp, _sz, _i, _sz, _i, _vp, _vp, _vp, _u64, _i, _vp]),
    "lc_level_sum_apply": (_i, [_vp, _sz, _i, _sz, _i, _vp, _u64, _i, _vp, _f, _f, _vp, _sz, _vp, _sz, _i, _i, _f, _vp]),
    "lc_container_bits": (_i, [_i]),
    "lc_status_string": (C.c_char_p, [_i]),
    "lc_stream_probe": (_i, [_i, _vp, _vp, _sz, _f, _vp]),
    "lc_version": (_i, []),
}

_lib = None


class LionCubError(RuntimeError):
    def __init__(self, name, status, text):
        super().__init__("%s failed with status %d (%s)" % (name, status, text))
        self.status = status


def load():
    """Load the HIP library (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        import torch  # noqa: F401  -- first, so that the process uses torch's HIP runtime
        if not os.path.exists(LIB_PATH):
            raise ImportError("%s is missing: build it with `python paper_2411_16462_amd/build.py`; "
                              "there is no fallback path" % LIB_PATH)
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def _ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if not x.is_cuda:
        raise ValueError("pointer arguments must be GPU tensors")
    return x.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def _call(name, check, *args):
    lib = load()
    rc = getattr(lib, name)(*args)
    if rc != LC_OK and check:
        raise LionCubError(name, rc, lib.lc_status_string(rc).decode())
    return rc


def lc_local_update_pack(g, g_stride_elems, g_dtype, m, m_stride_elems, W, n, beta1, update_m, beta2,
                         out_bits, q, q_stride_bytes, step, zero_rule, stream=None, check=True):
    return _call("lc_local_update_pack", check, _ptr(g), g_stride_elems, g_dtype, _ptr(m), m_stride_elems, W, n,
                 beta1, int(update_m), beta2, out_bits, _ptr(q), q_stride_bytes, step, zero_rule, _stream(stream))


def lc_vote_1bit(q, q_stride_words, W, n, vote_pos, vote_nz, step, tie_rule, stream=None, check=True):
    return _call("lc_vote_1bit", check, _ptr(q), q_stride_words, W, n, _ptr(vote_pos), _ptr(vote_nz), step,
                 tie_rule, _stream(stream))


def lc_pbit_sum_sign(q, q_stride_bytes, in_bits, W, n, p, sum_out, vote_pos, vote_nz, step, tie_rule,
                     stream=None, check=True):
    return _call("lc_pbit_sum_sign", check, _ptr(q), q_stride_bytes, in_bits, W, n, p, _ptr(sum_out),
                 _ptr(vote_pos), _ptr(vote_nz), step, tie_rule, _stream(stream))


def lc_apply_update(theta, vote_pos, vote_nz, n, lr, wd, m, m_stride_elems, g, g_stride_elems, g_dtype, n_m,
                    beta2, stream=None, check=True):
    return _call("lc_apply_update", check, _ptr(theta), _ptr(vote_pos), _ptr(vote_nz), n, lr, wd, _ptr(m),
                 m_stride_elems, _ptr(g), g_stride_elems, g_dtype, n_m, beta2, _stream(stream))


def lc_count_apply(k_fields, field_bits, n, total, step, tie_rule, theta, lr, wd, m, m_stride_elems, g, g_stride_elems,
                   g_dtype, n_m, beta2, stream=None, check=True):
    return _call("lc_count_apply", check, _ptr(k_fields), field_bits, n, total, step, tie_rule, _ptr(theta), lr, wd,
                 _ptr(m), m_stride_elems, _ptr(g), g_stride_elems, g_dtype, n_m, beta2, _stream(stream))


def lc_momentum_avg(m, m_stride_elems, W, n, stream=None, check=True):
    return _call("lc_momentum_avg", check, _ptr(m), m_stride_elems, W, n, _stream(stream))


def lc_momentum_divergence(m, m_stride_elems, W, n, max_std, stream=None, check=True):
    return _call("lc_momentum_divergence", check, _ptr(m), m_stride_elems, W, n, _ptr(max_std), _stream(stream))


def lc_momentum_divergence_groups(m, m_stride_elems, W, n, group_end64, n_groups, max_std, stream=None, check=True):
    return _call("lc_momentum_divergence_groups", check, _ptr(m), m_stride_elems, W, n, _ptr(group_end64), n_groups,
                 _ptr(max_std), _stream(stream))


def lc_momentum_sync_ranges(m, m_stride_elems, W, offsets, sizes, n_ranges, step, every, stream=None, check=True):
    """offsets / sizes: sequences of ints (host side), marshalled to size_t arrays."""
    off = (C.c_size_t * max(1, n_ranges))(*list(offsets)[:n_ranges]) if offsets is not None else None
    siz = (C.c_size_t * max(1, n_ranges))(*list(sizes)[:n_ranges]) if sizes is not None else None
    return _call("lc_momentum_sync_ranges", check, _ptr(m), m_stride_elems, W, off, siz, n_ranges, step, every,
                 _stream(stream))


def lc_vote_apply_1bit(q, q_stride_words, W, n, step, tie_rule, theta, lr, wd, m, m_stride_elems, g,
                       g_stride_elems, g_dtype, n_m, beta2, stream=None, check=True):
    return _call("lc_vote_apply_1bit", check, _ptr(q), q_stride_words, W, n, step, tie_rule, _ptr(theta), lr, wd,
                 _ptr(m), m_stride_elems, _ptr(g), g_stride_elems, g_dtype, n_m, beta2, _stream(stream))


def lc_vote_apply_1bit_groups(q, q_stride_words, W, n, step, tie_rule, theta, group_end64, group_lr, group_wd,
                              n_groups, stream=None, check=True):
    return _call("lc_vote_apply_1bit_groups", check, _ptr(q), q_stride_words, W, n, step, tie_rule, _ptr(theta),
                 _ptr(group_end64), _ptr(group_lr), _ptr(group_wd), n_groups, _stream(stream))


def lc_pbit_sum_apply(q, q_stride_bytes, in_bits, W, n, p, sum_out, step, tie_rule, theta, lr, wd, m,
                      m_stride_elems, g, g_stride_elems, g_dtype, n_m, beta2, stream=None, check=True):
    return _call("lc_pbit_sum_apply", check, _ptr(q), q_stride_bytes, in_bits, W, n, p, _ptr(sum_out), step,
                 tie_rule, _ptr(theta), lr, wd, _ptr(m), m_stride_elems, _ptr(g), g_stride_elems, g_dtype, n_m,
                 beta2, _stream(stream))


def lc_local_update_pack_ternary(g, g_stride_elems, g_dtype, m, m_stride_elems, W, n, beta1, update_m, beta2, pos, nz,
                                 q_stride_words, stream=None, check=True):
    return _call("lc_local_update_pack_ternary", check, _ptr(g), g_stride_elems, g_dtype, _ptr(m), m_stride_elems, W, n,
                 beta1, int(update_m), beta2, _ptr(pos), _ptr(nz), q_stride_words, _stream(stream))


def lc_vote_ternary(pos, nz, q_stride_words, W, n, vote_pos, vote_nz, stream=None, check=True):
    return _call("lc_vote_ternary", check, _ptr(pos), _ptr(nz), q_stride_words, W, n, _ptr(vote_pos), _ptr(vote_nz),
                 _stream(stream))


def lc_vote_apply_ternary(pos, nz, q_stride_words, W, n, theta, lr, wd, m, m_stride_elems, g, g_stride_elems, g_dtype,
                          n_m, beta2, stream=None, check=True):
    return _call("lc_vote_apply_ternary", check, _ptr(pos), _ptr(nz), q_stride_words, W, n, _ptr(theta), lr, wd,
                 _ptr(m), m_stride_elems, _ptr(g), g_stride_elems, g_dtype, n_m, beta2, _stream(stream))


def lc_pbit_sum_apply_groups(q, q_stride_bytes, in_bits, W, n, p, sum_out, step, tie_rule, theta, group_end64,
                             group_lr, group_wd, n_groups, stream=None, check=True):
    return _call("lc_pbit_sum_apply_groups", check, _ptr(q), q_stride_bytes, in_bits, W, n, p, _ptr(sum_out), step,
                 tie_rule, _ptr(theta), _ptr(group_end64), _ptr(group_lr), _ptr(group_wd), n_groups, _stream(stream))


def lc_vote_apply_ternary_groups(pos, nz, q_stride_words, W, n, theta, group_end64, group_lr, group_wd, n_groups,
                                 stream=None, check=True):
    return _call("lc_vote_apply_ternary_groups", check, _ptr(pos), _ptr(nz), q_stride_words, W, n, _ptr(theta),
                 _ptr(group_end64), _ptr(group_lr), _ptr(group_wd), n_groups, _stream(stream))


def lc_l1_mean_abs(g, g_stride_elems, g_dtype, m, m_stride_elems, W, n, beta1, mean_abs, workspace, stream=None,
                   check=True):
    return _call("lc_l1_mean_abs", check, _ptr(g), g_stride_elems, g_dtype, _ptr(m), m_stride_elems, W, n, beta1,
                 _ptr(mean_abs), _ptr(workspace), _stream(stream))


def lc_l1_mean_abs_static(g, g_stride_elems, g_dtype, m, m_stride_elems, W, n, beta1, mean_abs, stream=None, check=True):
    return _call("lc_l1_mean_abs_static", check, _ptr(g), g_stride_elems, g_dtype, _ptr(m), m_stride_elems, W, n,
                 beta1, _ptr(mean_abs), _stream(stream))


def lc_l1_quantize_pack(g, g_stride_elems, g_dtype, m, m_stride_elems, W, n, beta1, update_m, beta2, levels, mean_abs,
                        q, q_stride_bytes, stream=None, check=True):
    return _call("lc_l1_quantize_pack", check, _ptr(g), g_stride_elems, g_dtype, _ptr(m), m_stride_elems, W, n, beta1,
                 int(update_m), beta2, levels, _ptr(mean_abs), _ptr(q), q_stride_bytes, _stream(stream))


def lc_l1_groups_workspace_words(W, n_groups):
    return int(load().lc_l1_groups_workspace_words(W, n_groups))


def lc_l1_mean_abs_groups(g, g_stride_elems, g_dtype, m, m_stride_elems, W, n, beta1, group_end64, group_count,
                          n_groups, mean_abs, workspace, stream=None, check=True):
    return _call("lc_l1_mean_abs_groups", check, _ptr(g), g_stride_elems, g_dtype, _ptr(m), m_stride_elems, W, n,
                 beta1, _ptr(group_end64), _ptr(group_count), n_groups, _ptr(mean_abs), _ptr(workspace),
                 _stream(stream))


def lc_l1_quantize_pack_groups(g, g_stride_elems, g_dtype, m, m_stride_elems, W, n, beta1, update_m, beta2, levels,
                               group_end64, n_groups, mean_abs, q, q_stride_bytes, stream=None, check=True):
    return _call("lc_l1_quantize_pack_groups", check, _ptr(g), g_stride_elems, g_dtype, _ptr(m), m_stride_elems, W,
                 n, beta1, int(update_m), beta2, levels, _ptr(group_end64), n_groups, _ptr(mean_abs), _ptr(q),
                 q_stride_bytes, _stream(stream))


def lc_level_sum_apply_groups(q, q_stride_bytes, W, n, levels, sum_out, step, tie_rule, theta, group_end64, group_lr,
                              group_wd, n_groups, stream=None, check=True):
    return _call("lc_level_sum_apply_groups", check, _ptr(q), q_stride_bytes, W, n, levels, _ptr(sum_out), step,
                 tie_rule, _ptr(theta), _ptr(group_end64), _ptr(group_lr), _ptr(group_wd), n_groups,
                 _stream(stream))


def lc_level_sum_sign(q, q_stride_bytes, W, n, levels, sum_out, vote_pos, vote_nz, step, tie_rule, stream=None,
                      check=True):
    return _call("lc_level_sum_sign", check, _ptr(q), q_stride_bytes, W, n, levels, _ptr(sum_out), _ptr(vote_pos),
                 _ptr(vote_nz), step, tie_rule, _stream(stream))


def lc_level_sum_apply(q, q_stride_bytes, W, n, levels, sum_out, step, tie_rule, theta, lr, wd, m, m_stride_elems, g,
                       g_stride_elems, g_dtype, n_m, beta2, stream=None, check=True):
    return _call("lc_level_sum_apply", check, _ptr(q), q_stride_bytes, W, n, levels, _ptr(sum_out), step, tie_rule,
                 _ptr(theta), lr, wd, _ptr(m), m_stride_elems, _ptr(g), g_stride_elems, g_dtype, n_m, beta2,
                 _stream(stream))


def lc_container_bits(p):
    return load().lc_container_bits(p)


def lc_status_string(status):
    return load().lc_status_string(status).decode()


def lc_stream_probe(kind, a, b, n, s, stream=None, check=True):
    return _call("lc_stream_probe", check, kind, _ptr(a), _ptr(b), n, s, _stream(stream))


def lc_version():
    return load().lc_version()
