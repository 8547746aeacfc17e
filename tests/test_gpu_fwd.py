"""Forward parity: the HIP path against the fp64 oracle, element by element, on the same seeded bf16 inputs."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import nsa_sel_oracle as orc
from gpu_util import Case, TOL_O, assert_close, assert_lse_close, to_f64

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["tiny"] + wl.SMALL_NAMES)
def test_forward_matches_oracle(name):
    print("case", name, flush=True)
    w = wl.realise(wl.small(name) if name != "tiny" else wl.named("tiny"))
    c = Case(w, bwd=False)
    o, lse = c.forward()
    Q, K, V, _ = c.host_f64()
    O_ref, LSE_ref = orc.forward(Q, K, V, w.idx, w.cu_seqlens, causal=w.causal, block=w.block)
    assert_close("O", to_f64(o), O_ref, TOL_O)
    assert_lse_close(to_f64(lse), LSE_ref)


def test_forward_custom_scale_and_adversarial_rows():
    print("case adversarial", flush=True)
    w = wl.realise(wl.Workload("adv", [900, 300], hq=6, hkv=2, topk=10, seed=21))
    w.idx = wl.draw_adversarial_indices(np.random.default_rng(3), w.seqlens, w.hkv, w.topk)
    w.idx[100:140] = -1                                   # rows with nothing selected
    c = Case(w, bwd=False, scale=0.05)
    o, lse = c.forward()
    Q, K, V, _ = c.host_f64()
    O_ref, LSE_ref = orc.forward(Q, K, V, w.idx, w.cu_seqlens, causal=True, scale=0.05)
    assert_close("O", to_f64(o), O_ref, TOL_O)
    assert_lse_close(to_f64(lse), LSE_ref)
    assert np.all(to_f64(o)[100:140] == 0)


def test_profile_records_only_selected_kernels():
    """The event recorder brackets the launches of the selected kernel kinds only and resets on collect."""
    print("case profile select", flush=True)
    import paper_2508_18224_amd as nsa
    w = wl.realise(wl.small("g3_k1"))
    c = Case(w, bwd=False)
    c.forward()
    nsa.profile_select(["fwd_main", "index_hist"])
    nsa.profile_enable(64)
    c.forward()
    c.forward()
    got = {n: v for n, v in nsa.profile_collect().items() if v[1]}
    assert set(got) == {"fwd_main", "index_hist"} and got["fwd_main"][1] == 2 and got["fwd_main"][0] > 0
    nsa.profile_select(None)
    c.forward()
    every = {n for n, v in nsa.profile_collect().items() if v[1]}
    assert {"fwd_main", "fwd_dense", "index_dense", "index_scatter", "index_scan"} <= every   # fwd_dense: dense pairs + merge
    nsa.profile_enable(0)
    c.forward()
    assert not any(v[1] for v in nsa.profile_collect().values())
