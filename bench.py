#!/usr/bin/env python3
"""Benchmark of the Lion Cub compressed-update hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic optimizer state that
is already resident in HBM: every worker's local update + pack, the W-way aggregation,
the apply (and, where the workload asks for it, momentum averaging) -- all through the C
ABI of liblioncub.so.  Prints ONE JSON line.  Its headline (value, ms_per_step, roofline,
cpu_baseline) is the largest workload that runs the whole path, c3 (GPT-2-medium shapes,
16 workers, bf16 gradients, momentum averaging every step); the same line carries, under
"configs", one entry per other benchmark configuration -- c0 (once on one resident working
set, once rotating over eight), c1, c2, c4 with the majority vote and c4 with the p = 7 sum
of signs written as byte counts -- each with its step time and, per kernel, duration,
algorithmic bytes and fraction of the HBM peak.

Timing protocol.  Two copies of the workload's state are built (eight for the rotating c0
entry); after the warm-up every buffer the step writes is restored from a pristine copy,
then exactly K steps run back to back, alternating between the copies, between one
synchronisation and the next (ms_per_step = that wall clock / K).  Every call is also
bracketed by HIP events on the launch stream (torch's current stream): per kernel and per
step the mean, the median and the minimum over the K steps are reported, and the roofline
entry divides the dominant kernel's algorithmic bytes by its mean launch duration.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3|c0|c1|c2|c4|l1|t2]
                    [--others default|none|c0,c1,...] [--sum] [--split [--one-plane]]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published peak


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c3")
    ap.add_argument("--others", default="default",
                    help="further configurations timed after the headline and reported under \"configs\": a comma "
                         "list of c0, c0rot, c1, c2, c4, c4sum, l1, t2; \"default\" = all five benchmark "
                         "configurations when the headline is c3, none otherwise; \"none\"")
    ap.add_argument("--other-steps", type=int, default=10, help="timed steps of each further configuration")
    ap.add_argument("--copies", type=int, default=2, help="state copies the timed steps alternate between (>= 1)")
    ap.add_argument("--cpu-sample", type=int, default=1 << 27,
                    help="parameters in the oracle's all-threads sample (0: skip the CPU leg)")
    ap.add_argument("--cpu-sample-single", type=int, default=1 << 24,
                    help="parameters in the oracle's single-thread sample")
    ap.add_argument("--cpu-threads", type=int, default=0,
                    help="0 = the cores this process may use, capped at 16 (one GPU's share of the box)")
    ap.add_argument("--sum", action="store_true",
                    help="pre-packed workload (c4): the p = 7 sum of signs with the counts written as bytes "
                         "(lc_pbit_sum_apply on 1-bit rows) instead of the majority vote")
    ap.add_argument("--one-plane", action="store_true",
                    help="with --split: the 1-bit wire form -- ties take the alternating sign, one plane is "
                         "written (the re-pack before the allgather) and one plane is applied")
    ap.add_argument("--per-tensor", action="store_true",
                    help="1-bit and L1 workloads with a tensor list: one set of calls per tensor instead of one per "
                         "arena (shows the small-tensor launch overhead; not the headline configuration)")
    ap.add_argument("--groups", action="store_true",
                    help="workloads with a tensor list (c1, c2, c3, l1, t2): per-tensor learning rates (and, for L1, per-tensor "
                         "scales) through the group-table entry points, still one launch set for the arena")
    ap.add_argument("--divergence", action="store_true",
                    help="c1, c2, c3: also take the divergence of the workers' momenta in every step (one value, or "
                         "one per tensor with --groups), after the momentum update and before any averaging")
    ap.add_argument("--split", action="store_true",
                    help="pre-packed workload (c4): lc_vote_1bit then lc_apply_update, the two calls either side of "
                         "the allgather of the vote, instead of the fused lc_vote_apply_1bit")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step (for odd and for even iterations) into HIP graphs and time replays; "
                         "per-kernel timings are then not available and the roofline entry is for the whole step")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the bare streaming kernels (lc_stream_probe) that give the `ceilings` entry")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="BYTES",
                    help="also run one plain device copy of BYTES (read BYTES, write BYTES) before the steps: "
                         "the reference point for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    return ap.parse_args()


class Kernel:
    """One C-ABI call of the step with its algorithmic bytes and HIP-event timing."""

    def __init__(self, name, fn, alg_bytes):
        self.name, self.fn, self.alg_bytes = name, fn, alg_bytes
        self.events = []

    def launch(self, torch, timed):
        if timed:
            a = torch.cuda.Event(enable_timing=True)
            b = torch.cuda.Event(enable_timing=True)
            a.record()
            self.fn()
            b.record()
            self.events.append((a, b))
        else:
            self.fn()

    def times_ms(self):
        return [a.elapsed_time(b) for a, b in self.events]


def stats(xs):
    """mean, median and minimum of a list of durations"""
    xs = sorted(xs)
    k = len(xs)
    if not k:
        return {"mean": float("nan"), "median": float("nan"), "min": float("nan")}
    med = xs[k // 2] if k % 2 else 0.5 * (xs[k // 2 - 1] + xs[k // 2])
    return {"mean": sum(xs) / k, "median": med, "min": xs[0]}


def group_table(wl, torch, dev):
    """Device arrays of a per-tensor group table: segment ends in units of 64 elements and a
    rate / decay per tensor (matrices at the base rate, vectors -- biases, LayerNorm -- at 30x
    and without decay)."""
    ends, off = [], 0
    for _, sz in wl.tensors:
        off += sz
        ends.append(off // 64)
    is_vec = [sz < 8192 for _, sz in wl.tensors]
    end64 = torch.tensor(ends, dtype=torch.int32, device=dev)
    lr_t = torch.tensor([wl.lr * (30.0 if v else 1.0) for v in is_vec], dtype=torch.float32, device=dev)
    wd_t = torch.tensor([0.0 if v else wl.wd for v in is_vec], dtype=torch.float32, device=dev)
    return end64, lr_t, wd_t, len(ends)


def build_step(wl, torch, lc, synth, per_tensor=False, groups=False, split=False, variant="vote", one_plane=False,
               share=None, divergence=False):
    """Allocate the workload on cuda:0 and return (kernels, state, step counter) for one
    step.  state["rmw"] names the buffers a step writes in place.  share: a state dict of
    an earlier copy whose read-only packed rows are reused (pre-packed workload)."""
    dev = "cuda"
    n, W = wl.n, wl.W
    nw = (n + 63) // 64
    hp = dict(beta1=wl.beta1, beta2=wl.beta2, lr=wl.lr, wd=wl.wd)
    st = {"rmw": ["theta", "m"]}
    step_no = [1]
    kernels = []
    if wl.mode == "prepacked":
        q = share["q"] if share else synth.make_prepacked(n, W, seed=wl.seed, device=dev, agree=wl.agree)
        s1 = synth.make_state(n, 1, seed=wl.seed + 1, device=dev, g_scale=1.4e-3, noise=0.0)
        theta, m, g = s1["theta"], s1["m"], s1["g"]
        st.update(q=q, theta=theta, m=m, g=g)
        if split:
            # the two halves as a multi-GPU run would call them around the allgather of the
            # vote: planes out, then planes in.  one_plane: the 1-bit wire form (a tie takes
            # the alternating sign, so one plane carries the whole vote)
            pos = torch.zeros(synth.packed_row_words(nw), dtype=torch.int64, device=dev)
            nz = None if one_plane else torch.zeros(synth.packed_row_words(nw), dtype=torch.int64, device=dev)
            tie = lc.LC_TIE_ALT if one_plane else lc.LC_TIE_ZERO
            planes = 1 if one_plane else 2
            st.update(pos=pos, nz=nz)
            kernels.append(Kernel(
                "vote_1bit",
                lambda: lc.lc_vote_1bit(q, q.stride(0), W, n, pos, nz, step_no[0], tie),
                n * (W / 8 + planes / 8)))
            kernels.append(Kernel(
                "apply_update",
                lambda: lc.lc_apply_update(theta, pos, nz, n, hp["lr"], hp["wd"], m, m.stride(0), g, g.stride(0),
                                           lc.LC_F32, 1, hp["beta2"]),
                n * (planes / 8 + 8 + 8 + 4)))
            return kernels, st, step_no
        if variant == "sum":
            # the p-bit route on the same rows: K = sum of the W bits as one byte per element
            # (p = 7 holds 0..64), written out, then the sign of 2K - W is applied
            C = lc.lc_container_bits(wl.p)
            ksum = torch.zeros(synth.round_up(n * C // 8, 64), dtype=torch.uint8, device=dev)
            st.update(sum_out=ksum)
            kernels.append(Kernel(
                "pbit_sum_apply",
                lambda: lc.lc_pbit_sum_apply(q, q.stride(0) * 8, 1, W, n, wl.p, ksum, step_no[0], lc.LC_TIE_ZERO, theta,
                                             hp["lr"], hp["wd"], m, m.stride(0), g, g.stride(0), lc.LC_F32, 1,
                                             hp["beta2"]),
                n * (W / 8 + C / 8 + 8 + 8 + 4)))
            return kernels, st, step_no
        kernels.append(Kernel(
            "vote_apply_1bit",
            lambda: lc.lc_vote_apply_1bit(q, q.stride(0), W, n, step_no[0], lc.LC_TIE_ZERO, theta, hp["lr"], hp["wd"],
                                          m, m.stride(0), g, g.stride(0), lc.LC_F32, 1, hp["beta2"]),
            n * (W / 8 + 8 + 8 + 4)))
        return kernels, st, step_no
    s = synth.make_state(n, W, seed=wl.seed, device=dev, g_dtype=wl.g_dtype, noise=wl.noise, m_spread=wl.m_spread,
                         dist=wl.dist)
    theta, m, g = s["theta"], s["m"], s["g"]
    gd = lc.LC_BF16 if wl.g_dtype == "bf16" else lc.LC_F32
    gb = 2 if wl.g_dtype == "bf16" else 4
    st.update(theta=theta, m=m, g=g)
    if wl.mode == "1bit" and per_tensor and wl.tensors:
        q = torch.zeros((W, synth.packed_row_words(nw, W)), dtype=torch.int64, device=dev)
        st["q"] = q
        spans, off = [], 0
        for _, sz in wl.tensors:
            assert sz % 64 == 0
            spans.append((off, sz))
            off += sz

        def pack_all():
            for o, sz in spans:
                lc.lc_local_update_pack(g[:, o:], g.stride(0), gd, m[:, o:], m.stride(0), W, sz, hp["beta1"], 1,
                                        hp["beta2"], 1, q[:, o // 64:], q.stride(0) * 8, step_no[0], lc.LC_ZERO_ALT)

        def vote_all():
            for o, sz in spans:
                lc.lc_vote_apply_1bit(q[:, o // 64:], q.stride(0), W, sz, step_no[0], lc.LC_TIE_ZERO, theta[o:],
                                      hp["lr"], hp["wd"], None, 0, None, 0, lc.LC_F32, 0, hp["beta2"])
        kernels.append(Kernel("local_update_pack[per tensor]", pack_all, W * n * (4 + gb + 4 + 1 / 8)))
        kernels.append(Kernel("vote_apply_1bit[per tensor]", vote_all, n * (W / 8 + 8)))
    elif wl.mode == "1bit":
        q = torch.zeros((W, synth.packed_row_words(nw, W)), dtype=torch.int64, device=dev)
        st["q"] = q
        kernels.append(Kernel(
            "local_update_pack",
            lambda: lc.lc_local_update_pack(g, g.stride(0), gd, m, m.stride(0), W, n, hp["beta1"], 1, hp["beta2"], 1, q,
                                            q.stride(0) * 8, step_no[0], lc.LC_ZERO_ALT),
            W * n * (4 + gb + 4 + 1 / 8)))
        if groups and wl.tensors:
            end64, lr_t, wd_t, G = group_table(wl, torch, dev)
            st.update(end64=end64, lr_t=lr_t, wd_t=wd_t)
            kernels.append(Kernel(
                "vote_apply_1bit_groups",
                lambda: lc.lc_vote_apply_1bit_groups(q, q.stride(0), W, n, step_no[0], lc.LC_TIE_ZERO, theta, end64,
                                                     lr_t, wd_t, G),
                n * (W / 8 + 8)))
        else:
            kernels.append(Kernel(
                "vote_apply_1bit",
                lambda: lc.lc_vote_apply_1bit(q, q.stride(0), W, n, step_no[0], lc.LC_TIE_ZERO, theta, hp["lr"],
                                              hp["wd"], None, 0, None, 0, lc.LC_F32, 0, hp["beta2"]),
                n * (W / 8 + 8)))
    elif wl.mode == "ternary":
        pos = torch.zeros((W, synth.packed_row_words(nw, W)), dtype=torch.int64, device=dev)
        nz = torch.zeros((W, synth.packed_row_words(nw, W)), dtype=torch.int64, device=dev)
        st.update(pos=pos, nz=nz)
        kernels.append(Kernel(
            "local_update_pack_ternary",
            lambda: lc.lc_local_update_pack_ternary(g, g.stride(0), gd, m, m.stride(0), W, n, hp["beta1"], 1, hp["beta2"],
                                                    pos, nz, pos.stride(0)),
            W * n * (4 + gb + 4 + 2 / 8)))
        if groups and wl.tensors:
            end64, lr_t, wd_t, G = group_table(wl, torch, dev)
            st.update(end64=end64, lr_t=lr_t, wd_t=wd_t)
            kernels.append(Kernel(
                "vote_apply_ternary_groups",
                lambda: lc.lc_vote_apply_ternary_groups(pos, nz, pos.stride(0), W, n, theta, end64, lr_t, wd_t, G),
                n * (2 * W / 8 + 8)))
        else:
            kernels.append(Kernel(
                "vote_apply_ternary",
                lambda: lc.lc_vote_apply_ternary(pos, nz, pos.stride(0), W, n, theta, hp["lr"], hp["wd"], None, 0, None, 0,
                                                 lc.LC_F32, 0, hp["beta2"]),
                n * (2 * W / 8 + 8)))
    elif wl.mode == "l1":
        L = wl.levels
        q = torch.zeros((W, synth.round_up(n, 64)), dtype=torch.uint8, device=dev)
        sum_out = torch.zeros(synth.round_up(n, 64), dtype=torch.uint8, device=dev)
        mean = torch.zeros(W, dtype=torch.float64, device=dev)
        ws = torch.zeros(W * lc.LC_L1_WORKSPACE_WORDS, dtype=torch.int64, device=dev)
        st.update(q=q, sum_out=sum_out, mean_abs=mean)
        if per_tensor and wl.tensors:
            # one scale per tensor the slow way: three calls per tensor
            spans, off = [], 0
            for _, sz in wl.tensors:
                assert sz % 64 == 0
                spans.append((off, sz))
                off += sz
            mean_t = torch.zeros((len(spans), W), dtype=torch.float64, device=dev)
            st["mean_abs"] = mean_t

            def mean_all():
                for k, (o, sz) in enumerate(spans):
                    lc.lc_l1_mean_abs(g[:, o:], g.stride(0), gd, m[:, o:], m.stride(0), W, sz, hp["beta1"], mean_t[k], ws)

            def quant_all():
                for k, (o, sz) in enumerate(spans):
                    lc.lc_l1_quantize_pack(g[:, o:], g.stride(0), gd, m[:, o:], m.stride(0), W, sz, hp["beta1"], 1,
                                           hp["beta2"], L, mean_t[k], q[:, o:], q.stride(0))

            def sum_all():
                for o, sz in spans:
                    lc.lc_level_sum_apply(q[:, o:], q.stride(0), W, sz, L, sum_out[o:], step_no[0], lc.LC_TIE_ZERO,
                                          theta[o:], hp["lr"], hp["wd"], None, 0, None, 0, lc.LC_F32, 0, hp["beta2"])
            kernels.append(Kernel("l1_mean_abs[per tensor]", mean_all, W * n * (4 + gb)))
            kernels.append(Kernel("l1_quantize_pack[per tensor]", quant_all, W * n * (4 + gb + 4 + 1)))
            kernels.append(Kernel("level_sum_apply[per tensor]", sum_all, n * (W + 1 + 8)))
        elif groups and wl.tensors:
            # one scale, rate and decay per tensor, three launches for the whole arena
            end64, lr_t, wd_t, G = group_table(wl, torch, dev)
            mean_g = torch.zeros((W, G), dtype=torch.float64, device=dev)
            ws_g = torch.zeros(lc.lc_l1_groups_workspace_words(W, G), dtype=torch.int64, device=dev)
            st.update(end64=end64, lr_t=lr_t, wd_t=wd_t, mean_abs=mean_g)
            kernels.append(Kernel(
                "l1_mean_abs_groups",
                lambda: lc.lc_l1_mean_abs_groups(g, g.stride(0), gd, m, m.stride(0), W, n, hp["beta1"], end64, None, G,
                                                 mean_g, ws_g),
                W * n * (4 + gb)))
            kernels.append(Kernel(
                "l1_quantize_pack_groups",
                lambda: lc.lc_l1_quantize_pack_groups(g, g.stride(0), gd, m, m.stride(0), W, n, hp["beta1"], 1,
                                                      hp["beta2"], L, end64, G, mean_g, q, q.stride(0)),
                W * n * (4 + gb + 4 + 1)))
            kernels.append(Kernel(
                "level_sum_apply_groups",
                lambda: lc.lc_level_sum_apply_groups(q, q.stride(0), W, n, L, sum_out, step_no[0], lc.LC_TIE_ZERO, theta,
                                                     end64, lr_t, wd_t, G),
                n * (W + 1 + 8)))
        else:
            kernels.append(Kernel(
                "l1_mean_abs",
                lambda: lc.lc_l1_mean_abs(g, g.stride(0), gd, m, m.stride(0), W, n, hp["beta1"], mean, ws),
                W * n * (4 + gb)))
            kernels.append(Kernel(
                "l1_quantize_pack",
                lambda: lc.lc_l1_quantize_pack(g, g.stride(0), gd, m, m.stride(0), W, n, hp["beta1"], 1, hp["beta2"], L, mean,
                                               q, q.stride(0)),
                W * n * (4 + gb + 4 + 1)))
            kernels.append(Kernel(
                "level_sum_apply",
                lambda: lc.lc_level_sum_apply(q, q.stride(0), W, n, L, sum_out, step_no[0], lc.LC_TIE_ZERO, theta, hp["lr"],
                                              hp["wd"], None, 0, None, 0, lc.LC_F32, 0, hp["beta2"]),
                n * (W + 1 + 8)))
    else:
        C = lc.lc_container_bits(wl.p)
        fb = (n * C + 7) // 8
        q = torch.zeros((W, synth.round_up(fb, 64)), dtype=torch.uint8, device=dev)
        sum_out = torch.zeros(synth.round_up(fb, 64), dtype=torch.uint8, device=dev)
        st.update(q=q, sum_out=sum_out)
        kernels.append(Kernel(
            "local_update_pack",
            lambda: lc.lc_local_update_pack(g, g.stride(0), gd, m, m.stride(0), W, n, hp["beta1"], 1, hp["beta2"], C, q,
                                            q.stride(0), step_no[0], lc.LC_ZERO_ALT),
            W * n * (4 + gb + 4 + C / 8)))
        if groups and wl.tensors:
            end64, lr_t, wd_t, G = group_table(wl, torch, dev)
            st.update(end64=end64, lr_t=lr_t, wd_t=wd_t)
            kernels.append(Kernel(
                "pbit_sum_apply_groups",
                lambda: lc.lc_pbit_sum_apply_groups(q, q.stride(0), C, W, n, wl.p, sum_out, step_no[0], lc.LC_TIE_ZERO,
                                                    theta, end64, lr_t, wd_t, G),
                n * (W * C / 8 + C / 8 + 8)))
        else:
            kernels.append(Kernel(
                "pbit_sum_apply",
                lambda: lc.lc_pbit_sum_apply(q, q.stride(0), C, W, n, wl.p, sum_out, step_no[0], lc.LC_TIE_ZERO, theta,
                                             hp["lr"], hp["wd"], None, 0, None, 0, lc.LC_F32, 0, hp["beta2"]),
                n * (W * C / 8 + C / 8 + 8)))
    if divergence:
        # Section 5.1's metric, taken where a training loop would take it: after the momentum update, before
        # any averaging.  One double per call, or one per tensor with the group table.
        if groups and wl.tensors:
            if "end64" not in st:
                st["end64"] = group_table(wl, torch, dev)[0]
            d_end, d_out = st["end64"], torch.zeros(len(wl.tensors), dtype=torch.float64, device=dev)
            kernels.append(Kernel("momentum_divergence_groups",
                                  lambda: lc.lc_momentum_divergence_groups(m, m.stride(0), W, n, d_end, len(wl.tensors), d_out),
                                  n * W * 4))
        else:
            d_out = torch.zeros(1, dtype=torch.float64, device=dev)
            kernels.append(Kernel("momentum_divergence", lambda: lc.lc_momentum_divergence(m, m.stride(0), W, n, d_out),
                                  n * W * 4))
        st["max_std"] = d_out
    if wl.momentum_avg:
        kernels.append(Kernel("momentum_avg", lambda: lc.lc_momentum_avg(m, m.stride(0), W, n), n * W * 8))
    return kernels, st, step_no




def ceilings(torch, lc, n=(1 << 29) + 4160, reps=10):
    """What bare streaming kernels of the library's own shape reach on this device, measured in this run
    (lc_stream_probe on two buffers of n floats): context for the roofline fractions, which stay against the
    published peak.  Median of `reps` launches each, GB/s."""
    a = torch.randn(n, device="cuda")
    b = torch.randn(n, device="cuda")
    kinds = (("read", lc.LC_PROBE_READ, 4), ("write", lc.LC_PROBE_WRITE, 4), ("copy", lc.LC_PROBE_COPY, 8),
             ("scale_in_place", lc.LC_PROBE_SCALE, 8), ("read2_write1", lc.LC_PROBE_RMW2, 12))
    out = {"unit": "GB/s", "floats_per_buffer": n, "launches": reps}
    for name, kind, per in kinds:
        ts = []
        for i in range(reps + 3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            lc.lc_stream_probe(kind, a, b, n, 1.0)
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        out[name] = per * n / (stats(ts[3:])["median"] * 1e-3) / 1e9
    del a, b
    torch.cuda.empty_cache()
    return out


def cpu_baseline(wl, st, torch, sample, sample_single, threads):
    """The oracle, as it stands, on the first parameters of the same buffers: once on one
    thread (the first `sample_single` parameters) and once split into contiguous chunks over
    the host threads this process may use (the first `sample`; the C loops release the GIL)."""
    from concurrent.futures import ThreadPoolExecutor

    import numpy as np

    import oracle as orc
    n = min(wl.n, sample)
    n -= n % 64
    allowed = len(os.sched_getaffinity(0))
    cores = threads or min(16, allowed)
    kw = dict(beta1=wl.beta1, beta2=wl.beta2, lr=wl.lr, wd=wl.wd, step=1)
    theta = st["theta"][:n].cpu().numpy()
    if wl.mode == "prepacked":
        words = st["q"][:, : n // 64].cpu().numpy().view(np.uint64)
        m = st["m"][:, :n].cpu().numpy()
        g = st["g"][:, :n].cpu().numpy()

        def work(lo, hi):
            b = np.stack([orc.unpack_1bit(words[w, lo // 64: hi // 64], hi - lo) for w in range(wl.W)])
            K, S, u = orc.count_sign(b, 1, orc.TIE_ZERO)
            orc.apply(theta[lo:hi], u, wl.lr, wl.wd)
            orc.momentum(m[0, lo:hi], g[0, lo:hi], wl.beta2)
    else:
        m = st["m"][:, :n].cpu().numpy()
        if wl.g_dtype == "bf16":
            g = st["g"][:, :n].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
            gd = orc.BF16
        else:
            g = st["g"][:, :n].cpu().numpy()
            gd = orc.F32

        def work(lo, hi):
            if wl.mode == "1bit":
                r = orc.step_1bit(theta[lo:hi], m[:, lo:hi], g[:, lo:hi], g_dtype=gd, **kw)
            elif wl.mode == "ternary":
                kt = {k: v for k, v in kw.items() if k != "step"}
                r = orc.step_ternary(theta[lo:hi], m[:, lo:hi], g[:, lo:hi], g_dtype=gd, **kt)
            elif wl.mode == "l1":   # per-chunk scales: same work per element as per-call scales
                r = orc.step_l1(theta[lo:hi], m[:, lo:hi], g[:, lo:hi], L=wl.levels, g_dtype=gd, **kw)
            else:
                r = orc.step_pbit(theta[lo:hi], m[:, lo:hi], g[:, lo:hi], p=wl.p, g_dtype=gd, **kw)
            if wl.momentum_avg:
                orc.momentum_avg(r["m"].astype(np.float32))
    # (a) one thread, chunk after chunk
    n1 = min(n, sample_single)
    n1 -= n1 % 64
    chunk1 = 1 << 20
    t0 = time.perf_counter()
    for lo in range(0, n1, chunk1):
        work(lo, min(n1, lo + chunk1))
    dt1 = time.perf_counter() - t0
    # (b) contiguous chunks over the threads
    chunk = max(64, (n // (cores * 4)) // 64 * 64)
    spans = [(lo, min(n, lo + chunk)) for lo in range(0, n, chunk)]
    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=cores) as ex:
        list(ex.map(lambda s: work(*s), spans))
    dt = time.perf_counter() - t0
    return {"value": n / dt, "unit": "params/s", "cores": cores, "kind": "oracle",
            "host_cpus": os.cpu_count(), "cpus_allowed": allowed,
            "single_thread": {"value": n1 / dt1 if n1 else None, "unit": "params/s", "cores": 1,
                              "sample": "first %d params of %s, all %d workers, %.2f s" % (n1, wl.name, wl.W, dt1)},
            "sample": "first %d params of %s, all %d workers, %d chunks over %d threads, %.2f s"
                      % (n, wl.name, wl.W, len(spans), cores, dt)}


def read_traffic(workload, kernel):
    """HBM bytes per launch measured offline with rocprofv3 counters, if a summary that
    covers this workload and kernel has been committed under profiles/ (the workload's own
    file first, then its variants such as ..._p7_sum or ..._vote_then_apply)."""
    import glob
    own = os.path.join(ROOT, "profiles", "hbm_traffic_%s.txt" % workload)
    paths = [own] + sorted(p for p in glob.glob(os.path.join(ROOT, "profiles", "hbm_traffic_%s_*.txt" % workload)))
    for path in paths:
        if not os.path.exists(path):
            continue
        for line in open(path):
            parts = line.split("=")
            if len(parts) == 2 and parts[0].strip() == "traffic_bytes_per_launch." + kernel:
                return float(parts[1])
    return None


class Run:
    """`copies` copies of one workload's state and the timed steps over them."""

    def __init__(self, wl, torch, lc, synth, copies, **build_kw):
        self.wl, self.torch = wl, torch
        self.sets = []
        for _ in range(max(1, copies)):
            share = self.sets[0][1] if self.sets else None
            self.sets.append(build_step(wl, torch, lc, synth, share=share, **build_kw))
        st0 = self.sets[0][1]
        # every copy is drawn from the same seed, so one pristine copy restores them all
        self.pristine = {k: st0[k].clone() for k in st0["rmw"]}
        self.names = [k.name for k in self.sets[0][0]]
        self.step_events = []

    def restore(self):
        for kernels, st, step_no in self.sets:
            for k, src in self.pristine.items():
                st[k].copy_(src)
            step_no[0] = 1
            for kern in kernels:
                kern.events = []
        self.step_events = []

    def step(self, i, timed):
        kernels, _, step_no = self.sets[i % len(self.sets)]
        for k in kernels:
            k.launch(self.torch, timed)
        if timed:
            self.step_events.append((kernels[0].events[-1][0], kernels[-1].events[-1][1]))
        step_no[0] += 1

    def measure(self, warmup, steps):
        """warm-up, restore, then exactly `steps` steps between two synchronisations"""
        torch = self.torch
        for i in range(warmup):
            self.step(i, False)
        torch.cuda.synchronize()
        self.restore()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            self.step(i, True)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    def kernel_rows(self):
        rows = []
        for j, name in enumerate(self.names):
            ts = [t for kernels, _, _ in self.sets for t in kernels[j].times_ms()]
            b = self.sets[0][0][j].alg_bytes
            s = stats(ts)
            gbps = b / (s["mean"] * 1e-3) / 1e9
            rows.append({"kernel": name, "ms": s["mean"], "ms_median": s["median"], "ms_min": s["min"], "alg_bytes": b,
                         "achieved_GBps": gbps, "frac": gbps / HBM_PEAK_GBS,
                         "frac_median": b / (s["median"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
                         "traffic": read_traffic(self.wl.name, name)})
        return rows

    def step_stats(self):
        return stats([a.elapsed_time(b) for a, b in self.step_events])

    def step_bytes(self):
        return sum(k.alg_bytes for k in self.sets[0][0])


def calls_label(names):
    return ("per tensor" if any("[per tensor]" in x for x in names)
            else "one flat arena, per-tensor rates" if any(x.endswith("_groups") for x in names)
            else "vote, then apply from planes" if "apply_update" in names else "one flat arena")


# further configurations reported under "configs": workload, build arguments, state copies
OTHERS = {
    "c0": ("c0", {}, 1, "one resident working set (cache-resident, launch-bound: reported only)"),
    "c0rot": ("c0", {}, 8, "rotating over eight copies of the working set (480 MB: not cache-resident)"),
    "c1": ("c1", {}, 2, ""),
    "c2": ("c2", {}, 2, ""),
    "c4": ("c4", {}, 2, "majority vote + apply (28 B / param)"),
    "c4sum": ("c4", {"variant": "sum"}, 2, "p = 7 sum of signs written as byte counts + apply (29 B / param)"),
    "c4split": ("c4", {"split": True}, 2, "vote to two planes, then apply from the planes"),
    "c4split1": ("c4", {"split": True, "one_plane": True}, 2, "vote re-packed to one plane (ties alternate), then apply from it"),
    "l1": ("l1", {}, 2, ""),
    "t2": ("t2", {}, 2, ""),
}


def config_entry(run, ms_per_step, steps, note=""):
    wl = run.wl
    ss = run.step_stats()
    sb = run.step_bytes()
    out = {"workload": wl.name, "n_params": wl.n, "workers": wl.W, "steps": steps, "state_copies": len(run.sets),
           "ms_per_step": ms_per_step, "ms_per_step_median": ss["median"], "ms_per_step_min": ss["min"],
           "params_per_s": wl.n / (ms_per_step * 1e-3), "step_alg_bytes": sb,
           "step_frac_of_hbm_peak": sb / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, "kernels": run.kernel_rows()}
    if note:
        out["note"] = note
    return out


def main():
    args = parse()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (the W workers are simulated as W buffers in one GPU's HBM); "
                 "--gpus %d is not supported" % args.gpus)
    import torch

    import paper_2411_16462_amd as lc
    from paper_2411_16462_amd import synth
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    lc.load()
    torch.cuda.set_device(0)
    wl = synth.workload(args.workload)
    if args.divergence and wl.mode == "prepacked":
        sys.exit("bench.py: --divergence needs a workload with one momentum row per worker (c0 .. c3, l1, t2)")
    ceil = None if args.no_ceilings else ceilings(torch, lc)
    build_kw = dict(per_tensor=args.per_tensor, groups=args.groups, split=args.split,
                    variant="sum" if args.sum else "vote", one_plane=args.one_plane, divergence=args.divergence)
    run = Run(wl, torch, lc, synth, 1 if args.graph else args.copies, **build_kw)
    names = run.names                                   # what was built, not what was asked for
    torch.cuda.synchronize()
    if args.copy_calibration:
        src = torch.empty(args.copy_calibration, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.graph:
        kernels, st, step_no = run.sets[0]
        for i in range(args.warmup):
            run.step(i, False)
        torch.cuda.synchronize()
        run.restore()
        side = torch.cuda.Stream()
        graphs = {}
        with torch.cuda.stream(side):
            for parity in (1, 0):
                step_no[0] = 2 - parity                      # 1 (odd) or 2 (even): only the parity matters
                graphs[parity] = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graphs[parity], stream=side):
                    for k in kernels:
                        k.fn()
        torch.cuda.synchronize()
        for i in range(args.warmup):
            graphs[(i + 1) % 2].replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            graphs[(i + 1) % 2].replay()
        torch.cuda.synchronize()
        ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
        tot = run.step_bytes()
        gbps = tot / (ms_per_step * 1e-3) / 1e9
        per_kernel = [{"kernel": "whole step (graph replay)", "ms": ms_per_step, "ms_median": None, "ms_min": None,
                       "alg_bytes": tot, "achieved_GBps": gbps, "frac": gbps / HBM_PEAK_GBS, "traffic": None}]
        step_s = {"median": None, "min": None}
    else:
        ms_per_step = run.measure(args.warmup, args.steps)
        per_kernel = run.kernel_rows()
        step_s = run.step_stats()

    dom = max(per_kernel, key=lambda r: r["ms"])
    roofline = {"bound": "hbm", "kernel": dom["kernel"], "achieved": dom["achieved_GBps"], "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": dom["achieved_GBps"] / HBM_PEAK_GBS, "traffic": dom["traffic"],
                "alg_bytes_per_launch": dom["alg_bytes"], "avg_launch_ms": dom["ms"], "median_launch_ms": dom["ms_median"],
                "min_launch_ms": dom["ms_min"]}
    step_bytes = run.step_bytes()
    out = {
        "metric": "params/sec for Lion Cub step (pack+W-way vote+apply); % of HBM peak GB/s",
        "value": wl.n / (ms_per_step * 1e-3), "unit": "params/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "ms_per_step_median": step_s["median"],
        "ms_per_step_min": step_s["min"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32" if wl.g_dtype == "f32" else "f32 (bf16 gradients)", "data": "synthetic",
        "config": {"workload": wl.name, "n_params": wl.n, "workers": wl.W, "mode": wl.mode, "p": wl.p,
                   "g_dtype": wl.g_dtype, "momentum_avg": wl.momentum_avg, "levels": wl.levels,
                   "calls": calls_label(names), "state_copies": len(run.sets),
                   "launch": "hip graph replay" if args.graph else "stream"},
        "step_alg_bytes": step_bytes, "step_GBps": step_bytes / (ms_per_step * 1e-3) / 1e9,
        "step_frac_of_hbm_peak": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "roofline": roofline, "kernels": per_kernel,
    }
    if ceil is not None:
        # the bare kernel nearest to the dominant kernel's mix of reads and writes
        kind = "read2_write1" if "update_pack" in dom["kernel"] or "quantize" in dom["kernel"] else "copy"
        out["ceilings"] = ceil
        roofline.update(measured_ceiling=ceil[kind], measured_ceiling_kind=kind + " (lc_stream_probe, this run)",
                        frac_of_measured_ceiling=dom["achieved_GBps"] / ceil[kind])
    if args.cpu_sample > 0:
        out["cpu_baseline"] = cpu_baseline(wl, run.sets[0][1], torch, args.cpu_sample, args.cpu_sample_single,
                                           args.cpu_threads)
    else:
        out["cpu_baseline"] = None

    # the other benchmark configurations, one after the other, each freed before the next
    if args.others == "default":
        others = ["c0", "c0rot", "c1", "c2", "c4", "c4sum"] if wl.name.startswith("c3") and not (
            args.per_tensor or args.groups or args.graph or args.divergence) else []
    elif args.others in ("none", ""):
        others = []
    else:
        others = [x for x in args.others.split(",") if x]
    del run
    torch.cuda.empty_cache()
    configs = {}
    for key in others:
        if key not in OTHERS:
            sys.exit("bench.py: unknown configuration %r in --others" % key)
        wname, kw, copies, note = OTHERS[key]
        r = Run(synth.workload(wname), torch, lc, synth, copies, **kw)
        ms = r.measure(min(args.warmup, 3), args.other_steps)
        configs[key] = config_entry(r, ms, args.other_steps, note)
        del r
        torch.cuda.empty_cache()
    out["configs"] = configs
    if ceil is not None:  # every kernel also against the bare copy kernel of this run
        for rows in [out["kernels"]] + [e["kernels"] for e in configs.values()]:
            for k in rows:
                k["frac_of_measured_copy"] = k["achieved_GBps"] / ceil["copy"]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
