"""(Named to be collected after the other GPU tests.)  The C ABI from plain C: tests/c_client/step_client.c is compiled by gcc as C11 (so
include/lioncub.h is valid C, not only C++) and, on a GPU, run as a separate process with no
Python or torch inside; its results are compared with the CPU oracle."""
import importlib.util
import os
import subprocess

import numpy as np
import pytest

import oracle as orc
from conftest import ROOT
from harness import assert_close

_spec = importlib.util.spec_from_file_location("lc_c_client_build", os.path.join(ROOT, "tests", "c_client", "build.py"))
client_build = importlib.util.module_from_spec(_spec)
_spec.loader.exec_module(client_build)

HP = dict(beta1=0.9, beta2=0.99, lr=1e-4, wd=0.1)


def test_header_and_client_compile_as_c11():
    exe = client_build.build()
    assert os.access(exe, os.X_OK)
    out = subprocess.run([exe], capture_output=True, text=True)
    assert out.returncode == 1 and "usage" in out.stderr            # no GPU needed for the usage line


@pytest.mark.gpu
@pytest.mark.parametrize("n,W,step", [(100003, 5, 1), (64 * 300, 8, 2), (77, 3, 7)])
def test_plain_c_process_matches_the_oracle(n, W, step, tmp_path):
    exe = client_build.EXE
    if not os.path.exists(exe):            # normally built beforehand by __graft_entry__.build(); a 0.3 s gcc run otherwise
        client_build.build()
    rng = np.random.default_rng(4242 + n)
    theta = (rng.standard_normal(n) * 0.02).astype(np.float32)
    m = (rng.standard_normal((W, n)) * 1e-3).astype(np.float32)
    g = (rng.standard_normal((W, n)) * 1e-3).astype(np.float32)
    g[:, ::9] = 0
    m[:, ::9] = 0
    state, result = str(tmp_path / "state.bin"), str(tmp_path / "result.bin")
    with open(state, "wb") as f:
        np.array([n, W, step], np.uint64).tofile(f)
        theta.tofile(f)
        m.tofile(f)
        g.tofile(f)
    run = subprocess.run([exe, state, result], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0, run.stderr
    assert "planted error" in run.stdout          # the foreign pending error did not become the library's status
    nw = (n + 63) // 64
    with open(result, "rb") as f:
        theta1 = np.fromfile(f, np.float32, n)
        m1 = np.fromfile(f, np.float32, W * n).reshape(W, n)
        q = np.fromfile(f, np.uint64, W * nw).reshape(W, nw)
    ref = orc.step_1bit(theta, m, g, step=step, **HP)
    assert np.array_equal(q, ref["words"])
    assert_close(theta1, ref["theta"], "theta")
    assert_close(m1, ref["m"], "momentum")
    assert W % 2 == 1 or (ref["u"] == 0).any()                        # ties need an even worker count
