"""Backward parity: dQ, dK, dV of the HIP path against the fp64 oracle on the same seeded bf16 inputs."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import nsa_sel_oracle as orc
from gpu_util import Case, TOL_GRAD, assert_close, to_f64

pytestmark = pytest.mark.gpu


def _run(w, scale=0.0, oracle_scale=None):
    c = Case(w, bwd=True, scale=scale)
    o, lse = c.forward()
    dq, dk, dv = c.backward(o, lse)
    Q, K, V, dO = c.host_f64()
    rq, rk, rv = orc.backward(Q, K, V, dO, w.idx, w.cu_seqlens, causal=w.causal, scale=oracle_scale, block=w.block)
    assert_close("dQ", to_f64(dq), rq, TOL_GRAD)
    assert_close("dK", to_f64(dk), rk, TOL_GRAD)
    assert_close("dV", to_f64(dv), rv, TOL_GRAD)
    return c, (o, lse), (dq, dk, dv)


@pytest.mark.parametrize("name", ["tiny"] + wl.SMALL_NAMES)
def test_backward_matches_oracle(name):
    print("case", name, flush=True)
    _run(wl.realise(wl.small(name) if name != "tiny" else wl.named("tiny")))


def test_backward_long_list_splits_over_units_and_is_reproducible():
    """A sink list longer than one backward work unit: per-unit dK/dV partial sums, fixed-order reduction."""
    print("case long sink list", flush=True)
    w = wl.realise(wl.Workload("sink", [5000], hq=2, hkv=1, topk=4, sink=True, seed=31))
    c, (o, lse), (dq, dk, dv) = _run(w)
    dq2, dk2, dv2 = c.backward(o, lse)
    assert torch.equal(dk, dk2) and torch.equal(dv, dv2) and torch.equal(dq, dq2)


def test_backward_adversarial_rows_and_scale():
    print("case adversarial", flush=True)
    w = wl.realise(wl.Workload("adv", [900, 300], hq=6, hkv=2, topk=10, seed=21))
    w.idx = wl.draw_adversarial_indices(np.random.default_rng(3), w.seqlens, w.hkv, w.topk)
    w.idx[100:140] = -1
    _, _, (dq, _, _) = _run(w, scale=0.05, oracle_scale=0.05)
    assert np.all(to_f64(dq)[100:140] == 0)
