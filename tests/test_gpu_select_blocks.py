"""Block selection on the GPU (scores -> selection tensor) must equal the oracle's bit for bit: the decision is
taken on the fp32 scores as given on both sides, and the tie rule makes every row unique."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2508_18224_amd as nsa
import workloads as wl
from oracle import nsa_sel_oracle as orc
from oracle import topk_select_oracle as tko

pytestmark = pytest.mark.gpu


def _cu(seqlens):
    return np.concatenate([[0], np.cumsum(seqlens)]).astype(np.int32)


def _gpu_select(x, cu, topk, **kw):
    out = nsa.select_blocks(torch.from_numpy(x).cuda(), None if cu is None else torch.from_numpy(cu).cuda(), topk, **kw)
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("seqlens,hkv,topk,block,causal,n_sink,n_local,kind,stride", [
    ([2000], 2, 16, 64, True, 1, 2, "heavy", None),            # rows of 1 .. 32 blocks, 16-byte loads
    ([2000], 2, 16, 64, True, 1, 2, "ties", 33),               # odd stride: 4-byte loads
    ([700, 64, 1, 333, 1029], 3, 16, 64, True, 1, 2, "wild", None),
    ([900, 450], 2, 8, 64, False, 1, 1, "wild", 16),
    ([2100], 2, 8, 128, True, 1, 2, "ties", None),
    ([700, 129, 128, 1, 515], 2, 4, 128, True, 0, 1, "heavy", None),
    ([1500], 1, 32, 64, True, 2, 3, "ties", 24),
    ([777], 1, 1, 64, True, 0, 1, "heavy", None),
    ([777], 1, 1, 64, True, 0, 0, "heavy", None),
    ([1300], 2, 3, 64, True, 3, 3, "ties", None),              # more forced blocks than columns
    ([1300], 2, 12, 64, False, 0, 0, "wild", 21),              # plain top-k
])
def test_selection_bit_exact(seqlens, hkv, topk, block, causal, n_sink, n_local, kind, stride):
    print("case", seqlens, hkv, topk, block, causal, n_sink, n_local, kind, stride, flush=True)
    cu = _cu(seqlens)
    x = wl.draw_block_scores(31, seqlens, hkv, block, kind=kind, stride=stride, trap_future=causal)
    ref = tko.select_blocks(x, cu, topk, block=block, causal=causal, n_sink=n_sink, n_local=n_local)
    got = _gpu_select(x, cu, topk, block=block, causal=causal, n_sink=n_sink, n_local=n_local)
    assert np.array_equal(got, ref)


def test_single_sequence_without_cu():
    print("case no cu", flush=True)
    x = wl.draw_block_scores(32, [1000], 2, kind="heavy")
    ref = tko.select_blocks(x, _cu([1000]), 8)
    assert np.array_equal(_gpu_select(x, None, 8), ref)


@pytest.mark.parametrize("n_tokens,causal,kind,stride", [(70000, True, "ties", None), (140000, False, "heavy", 2190),
                                                         (140000, True, "ties", 2189)])
def test_rows_longer_than_one_chunk(n_tokens, causal, kind, stride):
    """More than 1024 visible blocks: the picks of several chunks are merged.  Oracle on sampled rows."""
    print("case multi-chunk", n_tokens, causal, kind, stride, flush=True)
    seqlens = [n_tokens]
    cu = _cu(seqlens)
    x = wl.draw_block_scores(33, seqlens, 1, kind=kind, stride=stride, trap_future=causal)
    rng = np.random.default_rng(5)
    tokens = np.unique(np.concatenate([rng.integers(0, n_tokens, 150), [0, 63, 64, 65535, 65536, 65599, 65600,
                                                                        n_tokens - 1]]))
    ref = tko.select_blocks(x, cu, 16, causal=causal, tokens=tokens)
    got = _gpu_select(x, cu, 16, causal=causal)
    assert np.array_equal(got[tokens], ref[tokens])


@pytest.mark.parametrize("n_tokens,causal,fill", [(70000, False, 0.25), (140000, True, -np.inf), (3000, True, np.nan)])
def test_all_scores_equal(n_tokens, causal, fill):
    """Every score the same: the bound the fast method derives keeps every block, so the row is handed to the general
    method (in rows of more than 128 blocks); the picks are then the smallest selectable block ids."""
    print("case all equal", n_tokens, causal, fill, flush=True)
    seqlens = [n_tokens]
    cu = _cu(seqlens)
    nb = -(-n_tokens // 64)
    x = np.full((n_tokens, 1, nb), fill, dtype=np.float32)
    rng = np.random.default_rng(7)
    tokens = np.unique(np.concatenate([rng.integers(0, n_tokens, 120), [0, 64, 2047, 2048, n_tokens - 1]]))
    ref = tko.select_blocks(x, cu, 16, causal=causal, tokens=tokens)
    got = _gpu_select(x, cu, 16, causal=causal)
    assert np.array_equal(got[tokens], ref[tokens])
    last = ref[n_tokens - 1, 0].tolist()
    assert last[:3] == ([0, (n_tokens - 1) // 64, (n_tokens - 1) // 64 - 1]) and last[3:] == list(range(1, 14))


def test_many_ties_at_the_bound():
    """A few distinct large scores over a sea of equal ones: more picks than distinct values, so the last picks are
    decided by block id among hundreds of equal scores."""
    print("case ties at the bound", flush=True)
    n_tokens, hkv = 100000, 2
    seqlens = [60000, 40000]
    cu = _cu(seqlens)
    rng = np.random.default_rng(8)
    x = np.ones((n_tokens, hkv, 938), dtype=np.float32)
    hot = rng.integers(0, 938, size=(n_tokens, hkv, 6))
    np.put_along_axis(x, hot, rng.random((n_tokens, hkv, 6)).astype(np.float32) + 2, axis=2)
    tokens = np.unique(np.concatenate([rng.integers(0, n_tokens, 150), [59999, 60000, n_tokens - 1]]))
    for causal in (True, False):
        ref = tko.select_blocks(x, cu, 16, causal=causal, tokens=tokens)
        got = _gpu_select(x, cu, 16, causal=causal)
        assert np.array_equal(got[tokens], ref[tokens])


def test_headline_shape_sampled_rows_and_properties():
    """N = 64K, 8 KV heads, 1024 blocks per row, top-16 with the sink and two local blocks forced: sampled rows
    against the oracle, and on every row the properties that hold at any size."""
    print("case headline selection", flush=True)
    T, hkv, topk = 65536, 8, 16
    seqlens = [T]
    cu = _cu(seqlens)
    x = wl.draw_block_scores(34, seqlens, hkv, kind="heavy")
    got = _gpu_select(x, cu, topk)
    tokens = np.unique(np.concatenate([np.random.default_rng(6).integers(0, T, 60), [0, 63, 64, 127, 128, T - 1]]))
    ref = tko.select_blocks(x, cu, topk, tokens=tokens)
    assert np.array_equal(got[tokens], ref[tokens])
    cur = (np.arange(T) // 64)[:, None, None]
    n_valid = np.minimum(cur + 1, topk)
    col = np.arange(topk)[None, None, :]
    assert np.array_equal(got >= 0, np.broadcast_to(col < n_valid, got.shape))
    assert (got <= cur).all()
    srt = np.sort(np.where(got < 0, -1 - col, got), axis=2)
    assert (np.diff(srt, axis=2) != 0).all()                      # no block twice in a row
    assert (got[:, :, 0] == 0).all()
    assert np.array_equal(got[64:, :, 1], np.broadcast_to(cur[64:, :, 0], (T - 64, hkv)))
    # free picks come in descending score order
    sc = np.take_along_axis(x, np.maximum(got, 0).astype(np.int64), axis=2)
    free = sc[4096:, :, 3:]
    assert (np.diff(free, axis=2) <= 0).all()


def test_selection_feeds_the_attention_path_on_the_device():
    """scores -> idx -> index inversion -> forward, all on the device, equals the oracle's forward on the oracle's idx."""
    print("case select then forward", flush=True)
    w = wl.realise(wl.small("g4"))
    cu = w.cu_seqlens
    x = wl.draw_block_scores(35, w.seqlens, w.hkv, kind="heavy")
    ref_idx = tko.select_blocks(x, cu, w.topk)
    cu_d = torch.from_numpy(cu).cuda()
    idx_d = nsa.select_blocks(torch.from_numpy(x).cuda(), cu_d, w.topk)
    attn = nsa.SelAttention(w.total_tokens, w.hq, w.hkv, w.topk, nseq=1, causal=True, bwd=False)
    from gpu_util import TOL_O, assert_close, dev_bf16, to_f64
    q, k, v = (dev_bf16(t) for t in (w.q, w.k, w.v))
    o, lse = attn.forward(q, k, v, idx_d, cu_d, rebuild_index=True)
    torch.cuda.synchronize()
    assert np.array_equal(idx_d.cpu().numpy(), ref_idx)
    Q, K, V = (wl.bf16_bits_to_f64(t) for t in (w.q, w.k, w.v))
    ro, _ = orc.forward(Q, K, V, ref_idx, cu, block=64, causal=True)
    assert_close("O", to_f64(o), ro, TOL_O)


def test_argument_errors():
    print("case select errors", flush=True)
    L = nsa.lib()
    x = torch.zeros(64, 1, 8, dtype=torch.float32, device="cuda")
    out = torch.empty(64, 1, 4, dtype=torch.int32, device="cuda")
    shape = nsa.Shape(64, 1, 1, 1, 128, 64, 4, 1, 0.0, 0)
    p = lambda t: C.c_void_p(t.data_ptr())
    assert L.nsa_sel_select_blocks(C.byref(shape), p(x), 8, None, 1, 2, None, None) == -1            # no output
    assert L.nsa_sel_select_blocks(C.byref(shape), None, 8, None, 1, 2, p(out), None) == 0            # no scores: forced blocks only
    torch.cuda.synchronize()
    assert out[63, 0].tolist() == [0, -1, -1, -1] and out[0, 0].tolist() == [0, -1, -1, -1]
    assert L.nsa_sel_select_blocks(C.byref(shape), p(x), 8, None, -1, 2, p(out), None) == -1
    assert L.nsa_sel_select_blocks(C.byref(shape), p(x), 0, None, 1, 2, p(out), None) == -2
    assert L.nsa_sel_select_blocks(C.byref(shape), p(x), 16385, None, 1, 2, p(out), None) == -2
    shape2 = nsa.Shape(64, 2, 1, 1, 128, 64, 4, 1, 0.0, 0)
    assert L.nsa_sel_select_blocks(C.byref(shape2), p(x), 8, None, 1, 2, p(out), None) == -1   # nseq > 1 needs cu
    shape3 = nsa.Shape(0, 1, 1, 1, 128, 64, 4, 1, 0.0, 0)
    assert L.nsa_sel_select_blocks(C.byref(shape3), p(x), 8, None, 1, 2, p(out), None) == 0     # nothing to do
