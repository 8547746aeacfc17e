"""Seeded random shapes (sequence mixes, head counts, top-k, block size, causal or not, adversarial rows) against the
oracle, forward and backward; plus unit-boundary cases where a list has exactly as many entries as a work unit."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import nsa_sel_oracle as orc
from gpu_util import Case, TOL_GRAD, TOL_O, assert_close, assert_lse_close, to_f64

pytestmark = pytest.mark.gpu


def _check(w, scale=0.0):
    c = Case(w, scale=scale)
    o, lse = c.forward()
    dq, dk, dv = c.backward(o, lse)
    Q, K, V, dO = c.host_f64()
    sc = None if scale == 0.0 else scale
    O_ref, LSE_ref = orc.forward(Q, K, V, w.idx, w.cu_seqlens, causal=w.causal, block=w.block, scale=sc)
    rq, rk, rv = orc.backward(Q, K, V, dO, w.idx, w.cu_seqlens, causal=w.causal, block=w.block, scale=sc)
    assert_close("O", to_f64(o), O_ref, TOL_O)
    assert_lse_close(to_f64(lse), LSE_ref)
    assert_close("dQ", to_f64(dq), rq, TOL_GRAD)
    assert_close("dK", to_f64(dk), rk, TOL_GRAD)
    assert_close("dV", to_f64(dv), rv, TOL_GRAD)


@pytest.mark.parametrize("seed", range(10))
def test_random_shape(seed):
    rng = np.random.default_rng(1000 + seed)
    nseq = int(rng.integers(1, 5))
    seqlens = [int(x) for x in rng.integers(1, 400, size=nseq)]
    hkv = int(rng.integers(1, 4))
    g = int(rng.integers(1, 9))
    block = int(rng.choice([64, 128]))
    topk = int(rng.integers(1, 9))
    causal = bool(rng.integers(0, 4) > 0)
    print("random case", seed, seqlens, hkv, g, block, topk, causal, flush=True)
    w = wl.Workload(f"r{seed}", seqlens, hq=hkv * g, hkv=hkv, topk=topk, causal=causal, sink=bool(rng.integers(0, 2)),
                    block=block, seed=seed)
    wl.realise(w)
    if rng.integers(0, 2):
        w.idx = wl.draw_adversarial_indices(rng, seqlens, hkv, topk, block=block)
    _check(w, scale=float(rng.choice([0.0, 0.11])))


@pytest.mark.parametrize("n_tokens,g", [(1024, 1), (1025, 1), (2048, 2), (2049, 1), (4096, 3), (4096 + 64, 1)])
def test_list_length_at_unit_boundaries(n_tokens, g):
    """Every token selects block 0 only: one list of exactly n_tokens entries, every other list empty (work units hold
    2048 entries, the backward keeps token ids in LDS 1024 entries at a time)."""
    print("boundary case", n_tokens, g, flush=True)
    w = wl.realise(wl.Workload("b", [n_tokens], hq=g, hkv=1, topk=2, seed=n_tokens))
    w.idx[:] = -1
    w.idx[:, :, 1] = 0
    _check(w)


@pytest.mark.parametrize("n_tokens,g,block", [(1, 1, 64), (2, 8, 64), (63, 3, 64), (64, 4, 128), (65, 1, 128), (129, 8, 128)])
def test_very_short_sequences(n_tokens, g, block):
    """Sequences shorter than, equal to and just past one block (one tile, one chunk, one work unit)."""
    print("short case", n_tokens, g, block, flush=True)
    w = wl.realise(wl.Workload("s", [n_tokens], hq=2 * g, hkv=2, topk=3, block=block, seed=n_tokens + g))
    _check(w)


def test_work_unit_size_changes_speed_not_results():
    """Every admissible unit size gives the same O, LSE and dQ bit for bit (a row's arithmetic does not depend on its
    tile neighbours) and dK/dV within the tolerance (their fp32 partial sums are split differently); the autotuner
    returns one of the candidates."""
    print("case unit sizes", flush=True)
    import paper_2508_18224_amd as nsa
    from gpu_util import Case, TOL_GRAD, assert_close, to_f64
    from oracle import nsa_sel_oracle as orc
    w = wl.realise(wl.Workload("units", [5000], hq=4, hkv=2, topk=6, sink=True, seed=91))
    c = Case(w)
    Q, K, V, dO = c.host_f64()
    _, rk, rv = orc.backward(Q, K, V, dO, w.idx, w.cu_seqlens)
    ref = None
    for unit in (256, 512, 1024, 2048):
        a = nsa.SelAttention(w.total_tokens, w.hq, w.hkv, w.topk, unit=unit)
        o, lse = a.forward(c.q, c.k, c.v, c.idx, c.cu)
        dq, dk, dv = a.backward(c.q, c.k, c.v, o, lse, c.do, c.cu)
        torch.cuda.synchronize()
        assert_close("dK", to_f64(dk), rk, TOL_GRAD)
        assert_close("dV", to_f64(dv), rv, TOL_GRAD)
        if ref is None:
            ref = (o, lse, dq)
        else:
            assert torch.equal(o, ref[0]) and torch.equal(lse, ref[1]) and torch.equal(dq, ref[2])
    best, timings = nsa.SelAttention.autotuned(c.q, c.k, c.v, c.idx, c.do, c.cu, topk=w.topk, reps=2)
    assert best.shape.unit in timings and len(timings) == 4
