"""Sliding window through the path (the `win` term of Eq. (2)): shape.window hides the keys u <= t - window and drops
selected blocks that lie wholly before the window; with the table of blocks a window can touch as idx, forward and
backward are softmax attention over the last `window` tokens.  Parity against the fp64 oracle."""
import numpy as np
import pytest
import torch

import paper_2508_18224_amd as nsa
import workloads as wl
from oracle import nsa_sel_oracle as orc
from oracle import topk_select_oracle as tko
from gpu_util import Case, TOL_GRAD, TOL_O, assert_close, assert_lse_close, to_f64

pytestmark = pytest.mark.gpu


def _oracle_window_table(seqlens, hkv, window, block=64):
    """The blocks a causal window of `window` tokens can touch, from the selection oracle: no sink, the
    R + 1 = ceil((window - 1) / block) + 1 most recent blocks forced, which leaves no free pick (scores are never read
    for a decision, so zeros serve)."""
    topk = -(-(window - 1) // block) + 1
    cu = np.concatenate([[0], np.cumsum(seqlens)]).astype(np.int64)
    nb = max(-(-L // block) for L in seqlens)
    scores = np.zeros((sum(seqlens), hkv, max(nb, 1)), dtype=np.float32)
    return tko.select_blocks(scores, cu, topk, block=block, causal=True, n_sink=0, n_local=topk)


@pytest.mark.parametrize("seqlens,hkv,window,block", [([2000], 2, 512, 64), ([700, 64, 1, 333, 1029], 3, 100, 64),
                                                      ([1500], 1, 1, 64), ([900, 450], 2, 64, 128),
                                                      ([3000], 1, 1000, 128), ([500], 2, 65, 64)])
def test_window_block_table_is_exact(seqlens, hkv, window, block):
    print("case window table", seqlens, hkv, window, block, flush=True)
    cu = np.concatenate([[0], np.cumsum(seqlens)]).astype(np.int32)
    got = nsa.window_blocks(sum(seqlens), hkv, window, torch.from_numpy(cu).cuda(), block=block)
    torch.cuda.synchronize()
    ref = _oracle_window_table(seqlens, hkv, window, block)
    assert np.array_equal(got.cpu().numpy(), ref)
    assert np.array_equal(wl.window_block_indices(seqlens, hkv, window, block), ref)   # the input generator agrees


def _run(w, window, idx=None, check_index=False):
    if idx is not None:
        w.idx = idx
        w.topk = idx.shape[2]
    c = Case(w, bwd=True, window=window)
    o, lse = c.forward()
    dq, dk, dv = c.backward(o, lse)
    Q, K, V, dO = c.host_f64()
    kw = dict(causal=True, block=w.block, window=window)
    rO, rL = orc.forward(Q, K, V, w.idx, w.cu_seqlens, **kw)
    assert_close("O", to_f64(o), rO, TOL_O)
    assert_lse_close(to_f64(lse), rL)
    rq, rk, rv = orc.backward(Q, K, V, dO, w.idx, w.cu_seqlens, **kw)
    assert_close("dQ", to_f64(dq), rq, TOL_GRAD)
    assert_close("dK", to_f64(dk), rk, TOL_GRAD)
    assert_close("dV", to_f64(dv), rv, TOL_GRAD)
    if check_index:
        cnt, off, qlist, qslot, vmask, bcap = c.attn.index_arrays()
        rc, ro, rl, rs, rvm = orc.invert_index(w.idx, w.cu_seqlens, block=w.block, window=window)
        assert np.array_equal(cnt[:, :rc.shape[1]], rc) and np.array_equal(qlist, rl) and np.array_equal(qslot, rs)
        assert np.array_equal(vmask, rvm)
    return c


@pytest.mark.parametrize("name,window", [("g4", 512), ("g4", 100), ("g1_varlen", 130), ("g8", 64), ("g7", 1),
                                         ("b128_g4", 512), ("b128_varlen", 200), ("g2_hkv5", 300)])
def test_window_attention_matches_oracle(name, window):
    """idx = the blocks the window can touch: sliding-window attention over the last `window` tokens."""
    print("case window", name, window, flush=True)
    w = wl.realise(wl.small(name))
    idx = wl.window_block_indices(w.seqlens, w.hkv, window, w.block)
    _run(w, window, idx=idx, check_index=True)


def test_window_with_arbitrary_selection():
    """A window on top of an ordinary selection: blocks wholly before the window are dropped by the inversion, the
    others are clipped; rows whose every selected block is out of the window give O = 0, LSE = -inf."""
    print("case window + selection", flush=True)
    w = wl.realise(wl.small("g4"))
    c = _run(w, 200, check_index=True)
    w2 = wl.realise(wl.Workload("sinkonly", [1000], hq=4, hkv=2, topk=1, sink=True, recent=0, seed=61))
    w2.idx[:] = 0                                         # only the sink block: out of the window from token 264 on
    c = _run(w2, 200)
    o, lse = c.forward()
    assert not to_f64(o)[300:].any() and np.isneginf(to_f64(lse)[300:]).all()


def test_window_table_from_the_device_feeds_the_path():
    print("case window chain", flush=True)
    w = wl.realise(wl.small("g4"))
    window = 300
    cu_d = torch.from_numpy(w.cu_seqlens).cuda()
    idx_d = nsa.window_blocks(w.total_tokens, w.hkv, window, cu_d)
    w.idx = idx_d.cpu().numpy()
    w.topk = w.idx.shape[2]
    assert np.array_equal(w.idx, _oracle_window_table(w.seqlens, w.hkv, window))
    _run(w, window)
