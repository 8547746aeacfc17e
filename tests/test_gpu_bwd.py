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


@pytest.mark.parametrize("seqlens,hq,hkv,topk", [
    ([2500], 3, 1, 3),            # g = 3: a sink list of 2500 entries = one full unit (two 1024-entry segments) + a second unit
    ([1300, 77, 129], 8, 1, 2),   # g = 8: 10400 rows in the sink list's unit, ragged last blocks, a 1-block sequence
    ([640], 5, 5, 8),             # g = 1, more picks than blocks: short lists, tiles with a single row
])
def test_backward_128_key_blocks_long_lists(seqlens, hq, hkv, topk):
    """(B_K, T) = (128, .): lists longer than the token ids one workgroup keeps resident, an odd and an even number of
    64-row tiles per segment, group sizes that do not divide the tile, and ragged last blocks."""
    print("case b128 long lists", seqlens, hq, hkv, topk, flush=True)
    w = wl.realise(wl.Workload("b128long", seqlens, hq=hq, hkv=hkv, topk=topk, sink=True, block=128, seed=77 + hq))
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


@pytest.mark.parametrize("hq,hkv", [(2, 1), (6, 2), (5, 1), (18, 3), (24, 4)])
def test_other_group_sizes(hq, hkv):
    """g = 2, 3, 5, 6 and kv-head counts that do not divide the number of XCDs."""
    print("case heads", hq, hkv, flush=True)
    _run(wl.realise(wl.Workload("g", [1111], hq=hq, hkv=hkv, topk=12, sink=True, recent=2, seed=100 + hq)))


def test_empty_sequences_in_a_packed_batch():
    """Zero-length sequences own no blocks and no tokens; their neighbours are unaffected."""
    print("case empty sequences", flush=True)
    w = wl.Workload("e", [300, 0, 0, 129, 0, 64, 1], hq=4, hkv=2, topk=5, seed=41)
    _run(wl.realise(w))


def test_two_calls_share_nothing_but_the_index():
    """Forward with a cached index (rebuild_index = 0) equals forward with a rebuild; backward twice is bit-equal."""
    print("case cached index", flush=True)
    w = wl.realise(wl.small("g4"))
    c = Case(w)
    o1, l1 = c.forward(rebuild=True)
    o2, l2 = c.forward(rebuild=False)
    assert torch.equal(o1, o2) and torch.equal(l1, l2)
    g1 = c.backward(o1, l1)
    g2 = c.backward(o1, l1)
    assert all(torch.equal(a, b) for a, b in zip(g1, g2))
