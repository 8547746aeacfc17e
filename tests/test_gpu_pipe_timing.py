"""The measuring build of the library (shader-clock stamps inside the pipelined 128-key backward kernel) gives the same
results as the product library, and its stamps are consistent: both wave roles of a workgroup live equally long."""
import os
import re
import subprocess
import sys

import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import Case

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CHILD = r"""
import sys, numpy as np, torch
sys.path.insert(0, sys.argv[1]); sys.path.insert(0, sys.argv[1] + "/tests")
from paper_2508_18224_amd import binding
from paper_2508_18224_amd.build import LIB_TIMING
binding._LIB_PATH = LIB_TIMING
import workloads as wl
from gpu_util import Case
c = Case(wl.realise(wl.small("b128_g4")))
o, lse = c.forward()
dq, dk, dv = c.backward(o, lse)
torch.cuda.synchronize()
np.savez(sys.argv[2], **{k: v.view(torch.int16).cpu().numpy() for k, v in dict(dq=dq, dk=dk, dv=dv).items()})
"""


def test_measuring_build_matches_the_product_library(tmp_path):
    print("case timing build parity", flush=True)
    out = str(tmp_path / "timing.npz")
    res = subprocess.run([sys.executable, "-c", CHILD, ROOT, out], capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    got = np.load(out)
    c = Case(wl.realise(wl.small("b128_g4")))
    o, lse = c.forward()
    dq, dk, dv = c.backward(o, lse)
    for name, ref in (("dq", dq), ("dk", dk), ("dv", dv)):
        assert np.array_equal(got[name], ref.view(torch.int16).cpu().numpy()), name


def test_phase_clocks_are_consistent():
    print("case pipe_timing module", flush=True)
    res = subprocess.run([sys.executable, "-m", "paper_2508_18224_amd.pipe_timing", "--workload", "grid_g4_b128_n8"],
                         cwd=ROOT, capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    totals = [float(x) for x in re.findall(r"^\s+(\d+)\s+total$", res.stdout, re.M)]
    assert len(totals) == 2 and totals[0] > 0, res.stdout
    assert abs(totals[0] - totals[1]) <= 0.02 * totals[0], res.stdout     # the two roles of a workgroup end together
