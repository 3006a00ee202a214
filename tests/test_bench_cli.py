"""Host-side checks of bench.py that need no GPU: the one-GPU rule, the workload table and
the bookkeeping of algorithmic bytes."""
import os
import subprocess
import sys

import bench
from paper_2411_16462_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_workload_table_matches_the_benchmark_configurations():
    w = {x.name.split("_")[0]: x for x in synth.workloads()}
    assert w["c0"].n == 1 << 20 and w["c0"].W == 4 and w["c0"].mode == "1bit"
    n_small = sum(s for _, s in synth.gpt2_tensors(768, 12))
    n_medium = sum(s for _, s in synth.gpt2_tensors(1024, 24))
    assert n_small == 124439808 and n_medium == 354823168                 # GPT-2 small / medium with tied head
    assert (w["c1"].n, w["c1"].W, w["c1"].mode) == (n_small, 8, "1bit")
    assert (w["c2"].n, w["c2"].W, w["c2"].mode, w["c2"].p, w["c2"].noise) == (n_small, 8, "pbit", 4, 0.5)
    assert (w["c3"].n, w["c3"].W, w["c3"].g_dtype, w["c3"].momentum_avg) == (n_medium, 16, "bf16", True)
    assert (w["c4"].n, w["c4"].W, w["c4"].mode, w["c4"].p, w["c4"].agree) == (1_300_000_000, 64, "prepacked", 7, 0.6)
    for x in w.values():
        assert (x.beta1, x.beta2, x.lr, x.wd) == (0.9, 0.99, 1e-4, 0.1)
    assert all(sz % 64 == 0 for _, sz in synth.gpt2_tensors(768, 12))      # tensors start on group boundaries
    assert len(synth.gpt2_tensors(768, 12)) == 148


def test_traffic_summaries_cover_the_dominant_kernels():
    """bench.py fills roofline.traffic from the committed counter summaries."""
    for name, kernel in (("c1_gpt2s_w8_1bit", "local_update_pack"), ("c2_gpt2s_w8_p4", "local_update_pack"),
                         ("c3_gpt2m_w16_bf16_1bit_mavg", "local_update_pack"),
                         ("c3_gpt2m_w16_bf16_1bit_mavg", "momentum_avg"),
                         ("c4_1p3b_w64_prepacked", "vote_apply_1bit"), ("c4_1p3b_w64_prepacked", "pbit_sum_apply"),
                         ("c4_1p3b_w64_prepacked", "vote_1bit"), ("l1_gpt2s_w8_l15", "l1_quantize_pack")):
        t = bench.read_traffic(name, kernel)
        assert t is not None and t > 1e9, (name, kernel)
    assert bench.read_traffic("no_such_workload", "x") is None


def test_default_headline_is_the_largest_full_path_workload():
    """No flags: c3 is the headline and the other benchmark configurations ride along."""
    old = sys.argv
    try:
        sys.argv = ["bench.py"]
        args = bench.parse()
    finally:
        sys.argv = old
    assert args.workload == "c3" and args.others == "default" and args.copies == 2 and args.steps == 20
    assert not args.no_ceilings and not args.divergence
    for key in ("c0", "c0rot", "c1", "c2", "c4", "c4sum"):
        wname, kw, copies, _ = bench.OTHERS[key]
        assert synth.workload(wname).name.startswith(key[:2])
    assert bench.OTHERS["c4sum"][1] == {"variant": "sum"} and bench.OTHERS["c0rot"][2] == 8
    assert bench.stats([3.0, 1.0, 2.0, 10.0]) == {"mean": 4.0, "median": 2.5, "min": 1.0}


def test_packed_row_strides_follow_the_measured_rule():
    """Few rows: an odd number of whole 128-byte lines; 32 and more rows: an odd number of 64-byte units."""
    for nw in (0, 1, 7, 16, 17, 1944372, 5544112, 20312500):
        few, many = synth.packed_row_words(nw, 8), synth.packed_row_words(nw, 64)
        assert few >= max(nw, 1) and few % 16 == 0 and (few // 16) % 2 == 1 and few - nw < 32
        assert many >= max(nw, 1) and many % 8 == 0 and (many // 8) % 2 == 1 and many - nw < 16
    assert synth.packed_row_words(20312500, 64) == 20312504 and synth.packed_row_words(5544112, 16) == 5544112
