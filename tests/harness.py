"""Test-side plumbing for the GPU parity tests: runs the HIP path through the Python
binding of the C ABI on torch device buffers and brings every stage back as numpy, and
runs the CPU oracle on the same inputs.  Holds no arithmetic of the method itself."""
import numpy as np
import torch

import oracle as orc
import paper_2411_16462_amd as lc
from paper_2411_16462_amd import synth

RTOL, ATOL = 1e-6, 1e-7          # fp32 outputs against the fp64 oracle
SENTINEL = 0x5A


def close(got, ref):
    """|got - ref| <= ATOL + RTOL * |ref|, element by element; returns the worst excess."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    err = np.abs(got - ref) - (ATOL + RTOL * np.abs(ref))
    return float(err.max()) if err.size else -1.0


def assert_close(got, ref, what):
    worst = close(got, ref)
    assert worst <= 0.0, "%s: tolerance exceeded by %.3e" % (what, worst)


def g_code(g):
    return lc.LC_BF16 if g.dtype == torch.bfloat16 else lc.LC_F32


def g_host(g):
    """Gradients for the oracle: float32 array, or the raw uint16 patterns of bf16."""
    if g.dtype == torch.bfloat16:
        return g.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return g.cpu().numpy()


def guarded(rows, nbytes, device, align=64):
    """uint8 (rows, stride) buffer filled with SENTINEL, stride > nbytes, rows aligned."""
    stride = synth.round_up(nbytes + 1, align) + align
    return torch.full((rows, stride), SENTINEL, dtype=torch.uint8, device=device)


def clone_rows(t):
    """Copy of a (W, n) row buffer that keeps the rows aligned (a plain clone() of the
    view would pack the rows back to back)."""
    out = torch.zeros((t.shape[0], synth.round_up(max(t.shape[1], 1), synth.ROW_ALIGN)), dtype=t.dtype,
                      device=t.device)[:, : t.shape[1]]
    out.copy_(t)
    return out


def words_of(buf, nw):
    """First nw 64-bit words of every row of a guarded uint8 buffer, as uint64 numpy."""
    return buf[:, : nw * 8].contiguous().cpu().numpy().view(np.uint64)


def untouched(buf, nbytes):
    return bool((buf[:, nbytes:] == SENTINEL).all().item())


class Case:
    """One synthetic optimizer state on the GPU plus host copies for the oracle."""

    def __init__(self, n, W, seed, g_dtype="f32", device="cuda", **kw):
        self.n, self.W = n, W
        st = synth.make_state(n, W, seed=seed, device=device, g_dtype=g_dtype, **kw)
        self.theta, self.m, self.g = st["theta"], st["m"], st["g"]
        self.device = device
        self.snapshot()

    def snapshot(self):
        self.theta0 = self.theta.cpu().numpy().copy()
        self.m0 = self.m.cpu().numpy().copy()
        self.g0 = g_host(self.g)

    @property
    def gd(self):
        return g_code(self.g)

    def oracle_gd(self):
        return orc.BF16 if self.g.dtype == torch.bfloat16 else orc.F32


def hip_update_pack(case, hp, step, out_bits=1, zero=lc.LC_ZERO_ALT, update_m=True, want_q=True):
    n, W = case.n, case.W
    nbytes = ((n + 63) // 64) * 8 if out_bits == 1 else (n * out_bits + 7) // 8
    q = guarded(W, nbytes, case.device) if want_q else None
    lc.lc_local_update_pack(case.g, case.g.stride(0), case.gd, case.m, case.m.stride(0), W, n, hp["beta1"],
                            update_m, hp["beta2"], out_bits, q, q.stride(0) if want_q else 0, step, zero)
    torch.cuda.synchronize()
    return q, nbytes


def oracle_step(case, hp, step, zero=orc.ZERO_ALT, tie=orc.TIE_ZERO, p=None):
    kw = dict(beta1=hp["beta1"], beta2=hp["beta2"], lr=hp["lr"], wd=hp["wd"], step=step, zero=zero, tie=tie,
              g_dtype=case.oracle_gd())
    if p is None:
        return orc.step_1bit(case.theta0, case.m0, case.g0, **kw)
    return orc.step_pbit(case.theta0, case.m0, case.g0, p=p, **kw)
