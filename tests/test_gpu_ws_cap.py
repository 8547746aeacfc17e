"""Capped workspaces (buffer reuse over head subsets, paper App. E): with a workspace that holds only some
of the KV heads the library works through the heads in several passes; the results must be bit-identical to
the single-pass ones (same arithmetic, same order) and the forward must still match the oracle."""
import numpy as np
import pytest
import torch

import paper_2508_18224_amd as nsa
import workloads as wl
from gpu_util import Case, TOL_O, assert_close, assert_lse_close, to_f64
from oracle import nsa_sel_oracle as oracle

pytestmark = pytest.mark.gpu


def _run(case):
    o, lse = case.forward()
    dq, dk, dv = case.backward(o, lse)
    return [x.clone() for x in (o, lse, dq, dk, dv)]


def _same_bits(a, b):
    if a.dtype == torch.bfloat16:
        return torch.equal(a.view(torch.int16), b.view(torch.int16))
    return torch.equal(a.view(torch.int32), b.view(torch.int32))


@pytest.mark.parametrize("name,heads", [("g2_hkv5", 1), ("g2_hkv5", 2), ("g1_varlen", 1), ("b128_g4", 1)])
def test_capped_workspace_matches_single_pass(name, heads):
    w = wl.realise(wl.small(name))
    full = Case(w)
    ref = _run(full)
    fmin, bmin = nsa.workspace_bytes_min(full.attn.shape)
    ffull, bfull, _ = nsa.workspace_bytes(full.attn.shape)
    assert fmin < ffull and bmin < bfull
    capped = Case(w)
    capped.attn = nsa.SelAttention(w.total_tokens, w.hq, w.hkv, w.topk, nseq=len(w.seqlens), causal=w.causal,
                                   block=w.block, ws_cap_bytes=heads * max(fmin, bmin), dense=True)
    assert capped.attn.fwd_ws.numel() < ffull and capped.attn.bwd_ws.numel() < bfull
    # poison the reused buffers so that a stale read from an earlier pass cannot go unnoticed
    capped.attn.fwd_ws.fill_(0x7F)
    capped.attn.bwd_ws.fill_(0x7F)
    got = _run(capped)
    for nm, a, b in zip(("O", "LSE", "dQ", "dK", "dV"), got, ref):
        assert _same_bits(a, b), f"{nm} differs between the capped and the full workspace"
    q, k, v, _ = full.host_f64()
    o_ref, lse_ref = oracle.forward(q, k, v, w.idx, w.cu_seqlens, block=w.block, causal=w.causal)
    assert_close("O", to_f64(got[0]), o_ref, TOL_O)
    assert_lse_close(to_f64(got[1]), lse_ref)


def test_workspace_below_minimum_is_rejected():
    w = wl.realise(wl.small("g2_hkv5"))
    case = Case(w)
    fmin, bmin = nsa.workspace_bytes_min(case.attn.shape)
    case.attn.fwd_ws = torch.empty(fmin - 256, dtype=torch.uint8, device="cuda")
    with pytest.raises(nsa.NsaSelError):
        case.forward()
