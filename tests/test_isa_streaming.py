"""Compile-time check (no GPU): the streaming kernels keep their non-temporal loads and
stores.  The compiler has been seen to drop the hint when a kernel's code took a certain
shape, which costs a quarter of the bandwidth without changing any result -- so the
generated gfx950 assembly is checked here."""
import os
import re
import subprocess

import pytest

from conftest import ROOT
from paper_2411_16462_amd import build as hip_build

CSRC = os.path.join(ROOT, "paper_2411_16462_amd", "csrc")


def device_asm(name, tmp_path):
    out = os.path.join(str(tmp_path), name + ".s")
    flags = [f for f in hip_build.FLAGS if f not in ("-fPIC", "-Wall", "-Wextra")]
    subprocess.check_call([hip_build.HIPCC, *flags, "-S", "--cuda-device-only", os.path.join(CSRC, name + ".hip"), "-o", out],
                          stderr=subprocess.DEVNULL)
    kernels, cur = {}, None
    for line in open(out):
        m = re.match(r"^(_ZN2lc\w+):", line)
        if m:
            cur = m.group(1)
            kernels[cur] = []
        elif cur and re.search(r"\bglobal_(load|store)_dwordx[24]\b", line):
            kernels[cur].append(line.strip())
        if line.startswith(".Lfunc_end"):
            cur = None
    return kernels


@pytest.mark.parametrize("source,pattern", [
    ("lc_update_pack", r"local_update_pack(_ternary)?_kernel"),
    ("lc_momentum_avg", r"momentum_(avg|avg_ranges|divergence)_kernel"),
    ("lc_l1", r"l1_(abs_sum|quantize_pack)_kernel"),
    ("lc_probe", r"stream_probe_kernelILi[0234]E"),               # kind 1 only writes: checked like the others below
])
def test_wide_accesses_are_non_temporal(source, pattern, tmp_path):
    kernels = {k: v for k, v in device_asm(source, tmp_path).items() if re.search(pattern, k)}
    assert kernels, "no kernel matched"
    for name, lines in kernels.items():
        wide = [l for l in lines if "dwordx4" in l]
        assert wide, name
        plain = [l for l in wide if not l.endswith(" nt")]
        assert not plain, "%s: %d of %d 16-byte accesses lost the non-temporal hint: %s" % (name, len(plain), len(wide), plain[:2])


def test_divergence_kernel_requests_every_row_before_it_uses_one(tmp_path):
    """The divergence kernel owes its speed to having all W <= CAP rows in flight at once (6.8 against 3.3 TB/s
    when the compiler interleaves loads and arithmetic): in each register-resident instance the first wait for a
    load must come after CAP 16-byte loads."""
    out = os.path.join(str(tmp_path), "avg.s")
    flags = [f for f in hip_build.FLAGS if f not in ("-fPIC", "-Wall", "-Wextra")]
    subprocess.check_call([hip_build.HIPCC, *flags, "-S", "--cuda-device-only", os.path.join(CSRC, "lc_momentum_avg.hip"), "-o", out],
                          stderr=subprocess.DEVNULL)
    seen, cur, loads, done = {}, None, 0, False
    for line in open(out):
        m = re.match(r"^_ZN2lc26momentum_divergence_kernelILi(\d+)ELb([01])EEE\w*:", line)
        if m:
            cur, loads, done = (int(m.group(1)), int(m.group(2))), 0, False
        elif cur and not done:
            if re.search(r"\bglobal_load_dwordx4\b", line):
                loads += 1
            elif re.search(r"\bs_waitcnt vmcnt", line) and loads >= 4:      # (a grouped instance first waits for its table)
                seen[cur] = loads
                done = True
        if line.startswith(".Lfunc_end"):
            cur = None
    assert set(seen) == {(c, g) for c in (4, 8, 16, 32, 64) for g in (0, 1)}, sorted(seen)
    for (cap, grouped), n_loads in seen.items():
        assert n_loads >= cap, "CAP = %d, grouped = %d: only %d loads before the first wait" % (cap, grouped, n_loads)


def test_aggregate_theta_and_momentum_streams_are_non_temporal(tmp_path):
    kernels = device_asm("lc_aggregate", tmp_path)
    apply_kernels = {k: v for k, v in kernels.items() if re.search(r"aggregate_kernelILi\d+ELi\dELb1", k)}
    assert len(apply_kernels) >= 12
    for name, lines in apply_kernels.items():
        stores = [l for l in lines if "store_dwordx4" in l]
        assert stores and all(l.endswith(" nt") for l in stores), name
        fields8 = re.search(r"aggregate_kernelILi8E", name)        # byte fields: 16-byte plain loads of packed rows
        loads = [l for l in lines if "load_dwordx4" in l and l.endswith(" nt")]
        tiles = 2 if name.endswith("ELi8EEEvNS_9AggParamsE") else 4  # 8 or 16 packed words per wave
        assert len(loads) >= tiles or fields8, name                 # the theta tiles (plus m, g streams)


def test_group_search_stays_on_the_scalar_unit(tmp_path):
    """The search through a group table must use scalar loads (scalar cache, own wait
    counter).  If the compiler cannot see that the tile base is uniform it turns them into
    vector loads that wait behind the wave's streaming loads -- same results, 75 % more
    time.  A scalar load whose base is not the kernel-argument pointer s[0:1] can only be a
    table access."""
    out = os.path.join(str(tmp_path), "agg.s")
    flags = [f for f in hip_build.FLAGS if f not in ("-fPIC", "-Wall", "-Wextra")]
    subprocess.check_call([hip_build.HIPCC, *flags, "-S", "--cuda-device-only", os.path.join(CSRC, "lc_aggregate.hip"), "-o", out],
                          stderr=subprocess.DEVNULL)
    table_loads, cur = {}, None
    for line in open(out):
        m = re.match(r"^(_ZN2lc\w+):", line)
        if m:
            cur = m.group(1)
            table_loads[cur] = 0
        elif cur and re.search(r"\bs_load_dword\s+s\d+,\s*s\[(?!0:1\])", line):
            table_loads[cur] += 1
        if line.startswith(".Lfunc_end"):
            cur = None
    grouped = {k: v for k, v in table_loads.items() if re.search(r"tile_apply_kernelILi\d+ELb[01]ELb1E", k)}
    assert len(grouped) >= 6
    for name, count in grouped.items():
        assert count >= 1, "%s: the group search lost its scalar loads" % name
    plain = {k: v for k, v in table_loads.items() if re.search(r"tile_apply_kernelILi\d+ELb[01]ELb0E", k)}
    assert plain and all(v == 0 for v in plain.values())                # and the pattern does single out the search
    general = {k: v for k, v in table_loads.items() if re.search(r"aggregate_kernelILi1ELi0ELb1ELb0ELb0E", k)}
    assert general and all(v >= 1 for v in general.values())
