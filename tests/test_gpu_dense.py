"""The dense forward route: (query tile, KV block) pairs that at least half of a tile's tokens keep are computed by the
query-tile-outer kernel, everything else by the gather route.  Whatever the split, O and LSE match the oracle; the
split itself is found by counting (never assumed), so the cases here make the detection partial: ragged tiles, rows
that drop the sink, occupancy around the threshold, tiles at sequence starts, packed batches."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import nsa_sel_oracle as orc
from gpu_util import Case, TOL_GRAD, TOL_O, assert_close, assert_lse_close, to_f64

pytestmark = pytest.mark.gpu


def _check(w, window=0, expect_dense=None, bwd=False):
    Q, K, V, dO = (wl.bf16_bits_to_f64(x) for x in (w.q, w.k, w.v, w.do))
    rO, rL = orc.forward(Q, K, V, w.idx, w.cu_seqlens, causal=w.causal, block=w.block, window=window)
    frac = {}
    for dense in (True, False):
        c = Case(w, bwd=bwd, window=window, dense=dense)
        o, lse = c.forward()
        assert_close(f"O dense={dense}", to_f64(o), rO, TOL_O)
        assert_lse_close(to_f64(lse), rL)
        flags = c.attn.dense_entries()
        frac[dense] = float(flags.mean()) if flags.size else 0.0
        # the inversion result does not depend on the routing
        cnt, off, qlist, qslot, vmask, bcap = c.attn.index_arrays()
        rc, ro, rl, rs, rvm = orc.invert_index(w.idx, w.cu_seqlens, block=w.block, causal=w.causal, window=window)
        assert np.array_equal(cnt[:, :rc.shape[1]], rc) and np.array_equal(qlist, rl) and np.array_equal(qslot, rs)
        if bwd:
            dq, dk, dv = c.backward(o, lse)
            rq, rk, rv = orc.backward(Q, K, V, dO, w.idx, w.cu_seqlens, causal=w.causal, block=w.block, window=window)
            assert_close("dQ", to_f64(dq), rq, TOL_GRAD)
            assert_close("dK", to_f64(dk), rk, TOL_GRAD)
            assert_close("dV", to_f64(dv), rv, TOL_GRAD)
    assert frac[False] == 0.0
    print("  dense share of the pairs:", round(frac[True], 3), flush=True)
    if expect_dense is not None:
        lo, hi = expect_dense
        assert lo <= frac[True] <= hi, frac
    return frac[True]


@pytest.mark.parametrize("name", wl.SMALL_NAMES)
def test_both_routes_match_the_oracle(name):
    print("case dense/gather", name, flush=True)
    _check(wl.realise(wl.small(name)), bwd=name in ("g4", "g1_varlen", "b128_g4"))


def test_sink_and_own_block_are_found_dense():
    """Sink + own block forced, 14 uniform picks: 2 of 16 slots of every late token, everything near the start."""
    print("case dense share", flush=True)
    w = wl.realise(wl.Workload("share", [4096], hq=8, hkv=2, topk=16, sink=True, seed=31))
    share = _check(w)
    assert 0.12 <= share <= 0.6


def test_rows_that_drop_the_sink_and_occupancy_around_the_threshold():
    print("case dense partial rows", flush=True)
    w = wl.realise(wl.Workload("partial", [1500, 700], hq=8, hkv=2, topk=8, sink=True, seed=32))
    rng = np.random.default_rng(5)
    T = w.total_tokens
    # every third token of the first KV head does not select the sink: the pair stays dense with a partial mask
    drop = (np.arange(T) % 3 == 0)
    w.idx[drop, 0, 0] = -1
    # tiles 8..15: block 2 kept by exactly 31, 32 or 33 of the 64 tokens (below, at and above one half)
    for n, tile in enumerate(range(8, 17)):
        keep = 31 + n % 3
        rows = np.arange(tile * 64, tile * 64 + 64)
        w.idx[rows, 1, 1] = np.where(np.arange(64) < keep, 2, w.idx[rows, 1, 1])
        clash = (w.idx[rows][:, 1, 2:] == 2).any(axis=1)            # keep rows duplicate-free for the recipe's sake
        w.idx[rows[clash], 1, 2:] = np.where(w.idx[rows[clash], 1, 2:] == 2, -1, w.idx[rows[clash], 1, 2:])
    # a tile whose first, middle and last tokens keep nothing at all
    w.idx[[1024, 1056, 1087], :, :] = -1
    _check(w, bwd=True)


def test_locality_picks_become_masked_dense_pairs():
    """Half of the free picks among the 8 most recent blocks (the g = 7 configuration's recipe): those pairs are kept
    by 7/8 of a tile's tokens and go dense with a row mask."""
    print("case dense locality", flush=True)
    w = wl.realise(wl.Workload("local", [3000], hq=7, hkv=1, topk=16, sink=True, local_picks=7, seed=33))
    share = _check(w, bwd=True)
    assert share >= 0.5


@pytest.mark.parametrize("seqlens,window,block", [([2000], 512, 64), ([700, 64, 1, 333, 1029], 100, 64),
                                                  ([900, 450], 300, 128), ([1500], 1, 64)])
def test_window_branch_is_all_dense(seqlens, window, block):
    print("case dense window", seqlens, window, block, flush=True)
    w = wl.realise(wl.Workload("win", seqlens, hq=4, hkv=2, topk=1, block=block, seed=34))
    w.idx = wl.window_block_indices(seqlens, 2, window, block)
    w.topk = w.idx.shape[2]
    _check(w, window=window, expect_dense=(0.9, 1.0), bwd=True)


def test_adversarial_selections_and_empty_rows():
    print("case dense adversarial", flush=True)
    w = wl.realise(wl.Workload("adv", [900, 300, 0, 65], hq=6, hkv=2, topk=10, seed=23))
    w.idx = wl.draw_adversarial_indices(np.random.default_rng(4), w.seqlens, w.hkv, w.topk)
    w.idx[100:140] = -1
    _check(w, bwd=True)
    w2 = wl.realise(wl.Workload("nc", [700, 300], hq=4, hkv=2, topk=12, causal=False, seed=35))
    w2.idx[:, :, 0] = 1                                            # every token of both sequences selects block 1
    _check(w2)


def test_dense_route_with_capped_workspace_is_bit_identical():
    print("case dense capped ws", flush=True)
    import paper_2508_18224_amd as nsa
    w = wl.realise(wl.small("g2_hkv5"))
    c = Case(w, bwd=False)
    o, lse = c.forward()
    c.attn = nsa.SelAttention(w.total_tokens, w.hq, w.hkv, w.topk, nseq=len(w.seqlens), causal=w.causal,
                              block=w.block, ws_cap_bytes=1, bwd=False, dense=True)
    o2, lse2 = c.forward()
    assert c.attn.dense_entries().any()
    assert torch.equal(o, o2) and torch.equal(lse, lse2)


def test_default_routing_policy():
    """shape.dense = 0: the dense route where it pays (g >= 2, or a window), the gather route at g = 1."""
    print("case dense policy", flush=True)
    import paper_2508_18224_amd as nsa
    big = wl.Workload("policy_g2", [9000], hq=4, hkv=2, topk=16, sink=True, seed=41)      # 288K triples
    big1 = wl.Workload("policy_g1", [9000, 300], hq=2, hkv=2, topk=16, seed=42)
    for name, window, expect in ((big, 0, True), (big1, 0, False), (big1, 100, True), ("g4", 0, False)):
        w = wl.realise(wl.small(name) if isinstance(name, str) else name)
        c = Case(w, bwd=False, window=window)
        c.attn = nsa.SelAttention(w.total_tokens, w.hq, w.hkv, w.topk, nseq=len(w.seqlens), causal=w.causal,
                                  block=w.block, window=window, bwd=False)        # dense=None: the library picks
        c.forward()
        assert bool(c.attn.dense_entries().any()) == expect, (name, window)
