"""The autograd wrapper is plumbing only: gradients that torch delivers through it are bit-identical to the library's
backward called directly, for the plain and the gated form."""
import numpy as np
import pytest
import torch

import paper_2508_18224_amd as nsa
import workloads as wl
from gpu_util import Case, dev_bf16

pytestmark = pytest.mark.gpu


def test_autograd_plain_equals_direct_calls():
    print("case autograd plain", flush=True)
    w = wl.realise(wl.small("g4"))
    c = Case(w)
    o_ref, lse_ref = c.forward()
    dq_ref, dk_ref, dv_ref = c.backward(o_ref, lse_ref)
    q, k, v = (t.clone().requires_grad_(True) for t in (c.q, c.k, c.v))
    o, lse = nsa.selected_attention(q, k, v, c.idx, c.attn, c.cu)
    o.backward(c.do)
    torch.cuda.synchronize()
    assert torch.equal(o, o_ref) and torch.equal(lse, lse_ref)
    assert torch.equal(q.grad, dq_ref) and torch.equal(k.grad, dk_ref) and torch.equal(v.grad, dv_ref)


def test_autograd_gated_equals_direct_calls():
    print("case autograd gated", flush=True)
    w = wl.realise(wl.small("g2_hkv5"))
    c = Case(w)
    T = w.total_tokens
    gate0 = torch.from_numpy(wl.draw_gates(5, T, w.hq)).cuda()
    acc0 = dev_bf16(wl.draw_other_branches(5, T, w.hq))
    out_ref, o_ref, lse_ref = c.attn.forward_gated(c.q, c.k, c.v, c.idx, gate0, acc0, c.cu)
    dq_ref, dk_ref, dv_ref, dg_ref = c.attn.backward_gated(c.q, c.k, c.v, o_ref, lse_ref, c.do, gate0, c.cu)
    q, k, v, gate, acc = (t.clone().requires_grad_(True) for t in (c.q, c.k, c.v, gate0, acc0))
    out = nsa.selected_attention(q, k, v, c.idx, c.attn, c.cu, gate=gate, o_acc=acc)
    out.backward(c.do)
    torch.cuda.synchronize()
    assert torch.equal(out, out_ref)
    assert torch.equal(q.grad, dq_ref) and torch.equal(k.grad, dk_ref) and torch.equal(v.grad, dv_ref)
    assert torch.equal(gate.grad, dg_ref) and torch.equal(acc.grad, c.do)


def test_readme_example_runs():
    """The usage shown in the README, on a small shape: selection, plain and gated calls, the window branch."""
    print("case readme example", flush=True)
    w = wl.realise(wl.small("g4"))
    total_tokens, hq, hkv, topk = w.total_tokens, w.hq, w.hkv, w.topk
    c = Case(w)
    q, k, v = (t.clone().requires_grad_(True) for t in (c.q, c.k, c.v))
    cu = c.cu
    scores = torch.from_numpy(wl.draw_block_scores(1, w.seqlens, hkv)).cuda()
    gate = torch.from_numpy(wl.draw_gates(1, total_tokens, hq)).cuda()
    o_acc = dev_bf16(wl.draw_other_branches(1, total_tokens, hq))
    attn = nsa.SelAttention(total_tokens, hq, hkv, topk, nseq=1, causal=True, block=64)
    idx = nsa.select_blocks(scores, cu, topk, n_sink=1, n_local=2)
    o, lse = nsa.selected_attention(q, k, v, idx, attn, cu)
    o.backward(c.do)
    out = nsa.selected_attention(q, k, v, idx, attn, cu, gate=gate, o_acc=o_acc)
    win = nsa.SelAttention(total_tokens, hq, hkv, topk=5, causal=True, block=128, window=512)
    o_win, _ = nsa.selected_attention(q, k, v, nsa.window_blocks(total_tokens, hkv, 512, cu, block=128), win, cu)
    torch.cuda.synchronize()
    for t in (o, out, o_win, q.grad, k.grad, v.grad):
        assert torch.isfinite(t.float()).all()
