"""Seeded synthetic inputs for the Lion Cub hot path.

This module only draws random buffers and lists tensor shapes.  It holds none of the
method's arithmetic (no interpolation, sign, packing, vote or update), so that the HIP
path and the CPU oracle can both be fed from it without sharing any of what they
compute.  The buffers stand in for the optimizer state of the paper's GPT-2-family
training runs (Appendix F.2 gives layer counts and widths); the paper's datasets and
trained weights are not needed because every kernel's memory traffic is independent
of the values.

Recipe (per workload): theta ~ N(0, 0.02^2) (GPT-2's initialisation scale),
a shared momentum m0 ~ N(0, (1e-3)^2) plus a per-worker deviation
m_w = m0 + m_spread * d_w with d_w ~ N(0, (1e-3)^2) (workers' momenta drift apart
because they are never synchronised, Section 5), and per-worker gradients
g_w = s + noise * e_w with a shared signal s and private noise e_w, both N(0, (1e-3)^2).
"""
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import torch

ROW_ALIGN = 64  # elements; keeps every worker's row 256-byte aligned for fp32
WORD_ALIGN = 16  # 64-bit words in a 128-byte line; see packed_row_words


def round_up(x: int, a: int) -> int:
    return (x + a - 1) // a * a


def packed_row_words(nw, W=1):
    """Row stride, in 64-bit words, for W rows of nw packed words.  Measured on the MI355X: the kernels
    that walk many rows per wave (32 and more) run fastest when the largest power of two that divides the
    stride is small -- 64 rows at c4's size: 5.85 ms at an odd multiple of 64 bytes, 6.05 at one of 128 or
    256, 6.25 at 512, 6.65 at 4 KiB -- so those get an odd number of 64-byte units; the few-worker kernel
    reads whole 128-byte lines of every row per workgroup and gains 2 % from rows that are whole lines, so
    fewer rows get an odd number of 128-byte lines."""
    unit = WORD_ALIGN // 2 if W >= 32 else WORD_ALIGN
    return ((max(nw, 1) + unit - 1) // unit | 1) * unit


def gpt2_tensors(d: int, n_layer: int, vocab: int = 50257, n_pos: int = 1024
                 ) -> List[Tuple[str, int]]:
    """(name, element count) of every parameter tensor of a GPT-2-style decoder with
    width d, n_layer blocks and a 4d MLP, in storage order."""
    t = [("wte", vocab * d), ("wpe", n_pos * d)]
    for i in range(n_layer):
        p = "h%d." % i
        t += [(p + "ln_1.w", d), (p + "ln_1.b", d),
              (p + "attn.c_attn.w", d * 3 * d), (p + "attn.c_attn.b", 3 * d),
              (p + "attn.c_proj.w", d * d), (p + "attn.c_proj.b", d),
              (p + "ln_2.w", d), (p + "ln_2.b", d),
              (p + "mlp.c_fc.w", d * 4 * d), (p + "mlp.c_fc.b", 4 * d),
              (p + "mlp.c_proj.w", 4 * d * d), (p + "mlp.c_proj.b", d)]
    t += [("ln_f.w", d), ("ln_f.b", d)]
    return t


@dataclass
class Workload:
    name: str
    n: int                      # parameters in the flat arena
    W: int                      # simulated workers
    mode: str                   # "1bit" | "pbit" | "prepacked" | "l1" | "ternary"
    p: int = 1                  # bits per summed field (pbit / prepacked-sum)
    levels: int = 0             # l1: levels on each side of zero (L = 15: Appendix F.1's 8-bit case)
    dist: str = "normal"        # gradient noise: "normal" | "laplace" (Section 4.1: updates look Laplacian)
    g_dtype: str = "f32"        # "f32" | "bf16"
    noise: float = 1.0          # g_w = s + noise * e_w
    m_spread: float = 0.05
    momentum_avg: bool = False
    agree: float = 0.6          # prepacked: P(worker bit == latent bit)
    seed: int = 0x11C0
    tensors: Optional[List[Tuple[str, int]]] = field(default=None, repr=False)
    beta1: float = 0.9
    beta2: float = 0.99
    lr: float = 1e-4
    wd: float = 0.1


def workloads() -> List[Workload]:
    small = gpt2_tensors(768, 12)
    medium = gpt2_tensors(1024, 24)
    n_small = sum(s for _, s in small)
    n_medium = sum(s for _, s in medium)
    return [
        Workload("c0_flat_1m_w4_1bit", 1 << 20, 4, "1bit", seed=0x11C0),
        Workload("c1_gpt2s_w8_1bit", n_small, 8, "1bit", tensors=small, seed=0x11C1),
        Workload("c2_gpt2s_w8_p4", n_small, 8, "pbit", p=4, noise=0.5, tensors=small,
                 seed=0x11C2),
        Workload("c3_gpt2m_w16_bf16_1bit_mavg", n_medium, 16, "1bit", g_dtype="bf16",
                 momentum_avg=True, tensors=medium, seed=0x11C3),
        Workload("c4_1p3b_w64_prepacked", 1_300_000_000, 64, "prepacked", p=7,
                 seed=0x11C4),
        # beyond the five benchmark configurations: the paper's 8-bit L1-quantised allreduce
        # among 8 workers (Appendix F.1), levels in [-15, 15], on the GPT-2-small shapes
        # ... and the ternary ("2-bit") wire format of Appendix B.1 on the same shapes
        Workload("t2_gpt2s_w8_ternary", n_small, 8, "ternary", tensors=small, seed=0x11C6),
        Workload("l1_gpt2s_w8_l15", n_small, 8, "l1", levels=15, dist="laplace", tensors=small,
                 seed=0x11C5),
    ]


def workload(name_or_index) -> Workload:
    ws = workloads()
    if isinstance(name_or_index, int):
        return ws[name_or_index]
    for w in ws:
        if w.name == name_or_index or w.name.split("_")[0] == name_or_index:
            return w
    raise KeyError(name_or_index)


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _rows(W: int, n: int, dtype, device) -> torch.Tensor:
    """(W, n) view whose rows start ROW_ALIGN-element aligned."""
    stride = round_up(max(n, 1), ROW_ALIGN)
    return torch.zeros((W, stride), dtype=dtype, device=device)[:, :n]


def _noise(n, gen, device, dist):
    if dist == "laplace":      # unit-variance Laplace by inverting its distribution function
        u = torch.rand(n, generator=gen, device=device) - 0.5
        return -torch.sign(u) * torch.log1p(-2.0 * u.abs().clamp(max=0.4999999)) * (0.5 ** 0.5)
    return torch.randn(n, generator=gen, device=device)


def make_state(n: int, W: int, *, seed: int, device="cpu", g_dtype: str = "f32",
               noise: float = 1.0, m_spread: float = 0.05, m_scale: float = 1e-3,
               g_scale: float = 1e-3, with_theta: bool = True, with_m: bool = True,
               dist: str = "normal"):
    """theta (n,), m (W, n) fp32 and g (W, n) fp32 or bf16, drawn as the module
    docstring states.  bf16 gradients are the fp32 draw rounded to nearest-even."""
    gen = _gen(device, seed)
    out = {}
    if with_theta:
        out["theta"] = torch.randn(n, generator=gen, device=device) * 0.02
    if with_m:
        m0 = torch.randn(n, generator=gen, device=device) * m_scale
        m = _rows(W, n, torch.float32, device)
        for w in range(W):
            m[w] = m0 + (m_spread * m_scale) * torch.randn(n, generator=gen, device=device)
        out["m"] = m
    s = _noise(n, gen, device, dist) * g_scale
    g = _rows(W, n, torch.bfloat16 if g_dtype == "bf16" else torch.float32, device)
    for w in range(W):
        gw = s + (noise * g_scale) * _noise(n, gen, device, dist)
        g[w] = gw.to(g.dtype)
    out["g"] = g
    return out


def biased_words(nw: int, prob_num: int, prob_bits: int, gen, device) -> torch.Tensor:
    """nw int64 words whose bits are independent and set with probability
    prob_num / 2**prob_bits.  Built from uniform random words by walking the binary
    expansion of the probability from its last digit: OR for a 1 digit, AND for a 0."""
    lo, hi = -(1 << 63), (1 << 63) - 1
    x = torch.zeros(nw, dtype=torch.int64, device=device)
    for k in range(prob_bits):
        r = torch.randint(lo, hi, (nw,), generator=gen, device=device, dtype=torch.int64)
        # randint's upper bound is exclusive: the single missing value 2^63-1 is immaterial
        if (prob_num >> k) & 1:
            x |= r
        else:
            x &= r
    return x


def make_prepacked(n: int, W: int, *, seed: int, device="cpu", agree: float = 0.6,
                   prob_bits: int = 10) -> torch.Tensor:
    """(W, ceil(n/64)) int64: worker w's 1-bit buffer equals a shared latent word with
    each bit flipped independently with probability 1 - agree (rounded to prob_bits
    binary digits).  Bits at positions >= n in the last word are zero."""
    gen = _gen(device, seed)
    nw = (n + 63) // 64
    lo, hi = -(1 << 63), (1 << 63) - 1
    latent = torch.randint(lo, hi, (nw,), generator=gen, device=device, dtype=torch.int64)
    flip_num = round((1.0 - agree) * (1 << prob_bits))
    q = torch.zeros((W, packed_row_words(nw, W)), dtype=torch.int64, device=device)[:, :nw]
    tail = n % 64
    for w in range(W):
        q[w] = latent ^ biased_words(nw, flip_num, prob_bits, gen, device)
        if tail and nw:
            keep = (1 << tail) - 1
            q[w, nw - 1] &= keep
    return q
