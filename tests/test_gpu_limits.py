"""The sizes at the edge of what the library accepts: the largest block count, thousands of packed sequences,
a call with no tokens at all."""
import numpy as np
import pytest
import torch

import paper_2508_18224_amd as nsa
import workloads as wl
from oracle import nsa_sel_oracle as orc
from gpu_util import BitsF64, Case, TOL_GRAD, TOL_O, TOL_LSE, assert_close, to_f64

pytestmark = pytest.mark.gpu


def _sampled(w, c, tokens):
    o, lse = c.forward()
    dq, dk, dv = c.backward(o, lse)
    Q, K, V, dO = (BitsF64(x) for x in (w.q, w.k, w.v, w.do))
    O_ref, LSE_ref = orc.forward(Q, K, V, w.idx, w.cu_seqlens, block=w.block, tokens=tokens)
    dQ_ref, _, _ = orc.backward(Q, K, V, dO, w.idx, w.cu_seqlens, block=w.block, tokens=tokens)
    sel = torch.tensor(tokens, device="cuda")
    assert_close("O", to_f64(o[sel]), O_ref[tokens], TOL_O)
    assert np.abs(to_f64(lse[sel]) - LSE_ref[tokens]).max() <= TOL_LSE
    assert_close("dQ", to_f64(dq[sel]), dQ_ref[tokens], TOL_GRAD)
    return dk, dv


def test_largest_block_count():
    """13 000 blocks of 64 tokens in one sequence, close to the limit the inversion's LDS tables set (one more
    thousand is refused): inversion bit-exact on whole lists, attention on sampled rows and one sampled KV block."""
    print("case block-count limit", flush=True)
    T = 13000 * 64
    assert nsa.lib().nsa_sel_workspace_bytes(nsa.Shape(14000 * 64, 1, 1, 1, 128, 64, 3, 1, 0.0, 0), None, None, None) == -2
    w = wl.realise(wl.Workload("limit", [T], hq=1, hkv=1, topk=3, sink=True, seed=81))
    c = Case(w)
    tokens = sorted({0, 63, 64, T - 1, *[int(x) for x in np.random.default_rng(1).integers(0, T, 10)]})
    dk, dv = _sampled(w, c, tokens)
    cnt, off, qlist, qslot, vmask, bcap = c.attn.index_arrays()
    rc, ro, rl, rs, rv = orc.invert_index(w.idx, w.cu_seqlens)
    assert np.array_equal(cnt[:, :rc.shape[1]], rc) and np.array_equal(qlist, rl) and np.array_equal(qslot, rs)
    Q, K, V, dO = (BitsF64(x) for x in (w.q, w.k, w.v, w.do))
    (dKb, dVb), = orc.backward_kv_blocks(Q, K, V, dO, w.idx, w.cu_seqlens, [(0, 0, 12999)])
    assert_close("dK last block", to_f64(dk[12999 * 64:, 0]), dKb, TOL_GRAD)
    assert_close("dV last block", to_f64(dv[12999 * 64:, 0]), dVb, TOL_GRAD)


def test_thousands_of_packed_sequences():
    """2 500 sequences of 1 .. 130 tokens (most shorter than a block, some empty): every sequence owns its blocks."""
    print("case many sequences", flush=True)
    rng = np.random.default_rng(82)
    seqlens = [int(x) for x in rng.integers(0, 131, 2500)]
    w = wl.realise(wl.Workload("many", seqlens, hq=4, hkv=2, topk=4, seed=82))
    T = w.total_tokens
    c = Case(w)
    tokens = sorted({0, T - 1, *[int(x) for x in rng.integers(0, T, 300)]})
    _sampled(w, c, tokens)
    cnt, off, qlist, qslot, vmask, bcap = c.attn.index_arrays()
    rc, ro, rl, rs, rv = orc.invert_index(w.idx, w.cu_seqlens)
    assert np.array_equal(cnt[:, :rc.shape[1]], rc) and np.array_equal(qlist, rl) and np.array_equal(vmask, rv)


def test_no_tokens_at_all():
    print("case zero tokens", flush=True)
    attn = nsa.SelAttention(0, 4, 2, 8, nseq=1)
    import ctypes as C
    L = nsa.lib()
    assert attn.fwd_ws.numel() == 0                       # a zero-byte workspace has no address
    rc = L.nsa_sel_build_index(C.byref(attn.shape), None, None, None, 0, None)
    assert rc == 0
    rc = L.nsa_sel_fwd(C.byref(attn.shape), None, None, None, None, None, 1, None, 0, None, None, None, 0, None)
    assert rc == 0
    rc = L.nsa_sel_bwd(C.byref(attn.shape), None, None, None, None, None, None, None, None, 0, None, None, None, None,
                       0, None)
    assert rc == 0
    torch.cuda.synchronize()
