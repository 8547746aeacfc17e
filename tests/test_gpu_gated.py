"""Gated combination fused into the path (Eq. (2)): O_out = O_acc + gate * O in the merge kernel, and in the backward
the gate folded into the per-row log-sum-exp, against the fp64 oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

import paper_2508_18224_amd as nsa
import workloads as wl
from oracle import nsa_sel_oracle as orc
from gpu_util import Case, TOL_GRAD, TOL_O, assert_close, assert_dgate_close, dev_bf16, to_f64

pytestmark = pytest.mark.gpu


def _gated(w, with_acc=True, in_place=False, ws_cap=None):
    c = Case(w, bwd=True)
    if ws_cap is not None:
        c.attn = nsa.SelAttention(w.total_tokens, w.hq, w.hkv, w.topk, nseq=len(w.seqlens), causal=w.causal,
                                  block=w.block, ws_cap_bytes=ws_cap)
    T = w.total_tokens
    gate = wl.draw_gates(w.seed, T, w.hq)
    acc_bits = wl.draw_other_branches(w.seed, T, w.hq) if with_acc else None
    gate_d = torch.from_numpy(gate).cuda()
    acc_d = dev_bf16(acc_bits) if with_acc else None
    out_buf = acc_d.clone() if (with_acc and in_place) else None
    o_out, o, lse = c.attn.forward_gated(c.q, c.k, c.v, c.idx, gate_d, out_buf if in_place else acc_d, c.cu,
                                         out=out_buf)
    torch.cuda.synchronize()
    o_plain, lse_plain = c.forward()
    assert torch.equal(o, o_plain) and torch.equal(lse, lse_plain)           # the ungated outputs are untouched
    Q, K, V, dO = c.host_f64()
    rO, _ = orc.forward(Q, K, V, w.idx, w.cu_seqlens, causal=w.causal, block=w.block)
    racc = wl.bf16_bits_to_f64(acc_bits) if with_acc else None
    assert_close("O_out", to_f64(o_out), orc.gated_forward(rO, gate.astype(np.float64), racc), TOL_O)
    dq, dk, dv, dgate = c.attn.backward_gated(c.q, c.k, c.v, o, lse, c.do, gate_d, c.cu)
    torch.cuda.synchronize()
    rq, rk, rv, rg = orc.gated_backward(Q, K, V, dO, gate.astype(np.float64), w.idx, w.cu_seqlens, causal=w.causal,
                                        block=w.block)
    assert_close("dQ", to_f64(dq), rq, TOL_GRAD)
    assert_close("dK", to_f64(dk), rk, TOL_GRAD)
    assert_close("dV", to_f64(dv), rv, TOL_GRAD)
    assert_dgate_close("dgate", to_f64(dgate), dO, rO)
    assert np.allclose(rg, (dO * rO).sum(axis=2))
    off = gate == 0.0
    assert off.any() and not to_f64(dq)[off].any()                              # a closed gate passes no gradient
    return c


@pytest.mark.parametrize("name", ["g4", "g1_varlen", "g2_noncausal", "b128_g4", "g2_hkv5"])
def test_gated_matches_oracle(name):
    print("case gated", name, flush=True)
    _gated(wl.realise(wl.small(name)))


def test_gated_without_other_branches_and_in_place():
    print("case gated no acc / in place", flush=True)
    _gated(wl.realise(wl.small("g8")), with_acc=False)
    _gated(wl.realise(wl.small("g7")), in_place=True)


def test_gated_with_capped_workspace():
    """One KV head per pass: the merge of every pass applies the gate to its own heads."""
    print("case gated capped ws", flush=True)
    _gated(wl.realise(wl.small("g2_hkv5")), ws_cap=1)    # clamped up to the library's minimum


def test_unit_gate_reproduces_the_plain_output_bit_for_bit():
    print("case unit gate", flush=True)
    w = wl.realise(wl.small("g4"))
    c = Case(w, bwd=True)
    ones = torch.ones(w.total_tokens, w.hq, dtype=torch.float32, device="cuda")
    o_out, o, lse = c.attn.forward_gated(c.q, c.k, c.v, c.idx, ones, None, c.cu)
    dq, dk, dv, dgate = c.attn.backward_gated(c.q, c.k, c.v, o, lse, c.do, ones, c.cu)
    pq, pk, pv = c.backward(o, lse)
    assert torch.equal(o_out, o)
    assert torch.equal(dq, pq) and torch.equal(dk, pk) and torch.equal(dv, pv)


def test_gated_argument_errors():
    print("case gated errors", flush=True)
    w = wl.realise(wl.small("g3_k1"))
    c = Case(w, bwd=True)
    gate = torch.ones(w.total_tokens, w.hq, dtype=torch.float32, device="cuda")
    o, lse = c.forward()
    with pytest.raises(nsa.NsaSelError):
        c.attn.forward_gated(c.q, c.k, c.v, c.idx, None, None, c.cu)           # no gate
    with pytest.raises(nsa.NsaSelError):
        c.attn.backward_gated(c.q, c.k, c.v, o, lse, c.do, None, c.cu)         # no gate
    # O_out must not be the ungated output buffer
    import ctypes as C
    p = lambda t: C.c_void_p(t.data_ptr())
    a = c.attn
    rc = nsa.lib().nsa_sel_fwd_gated(C.byref(a.shape), p(c.q), p(c.k), p(c.v), p(c.idx), p(c.cu), 1, p(a.index_ws),
                                     a.index_ws.numel(), p(o), p(lse), p(gate), None, p(o), p(a.fwd_ws),
                                     a.fwd_ws.numel(), None)
    assert rc == -1


def test_selected_and_window_branches_gated_into_one_output():
    """Eq. (2) with two of its three branches from this library: out = acc + tau_sel * sel + tau_win * win, the second
    call accumulating in place into the first one's output; gradients of each branch from its own backward."""
    print("case two branches", flush=True)
    w = wl.realise(wl.small("g4"))
    window = 200
    T = w.total_tokens
    c_sel = Case(w, bwd=True)
    w_win = wl.realise(wl.small("g4"))
    w_win.idx = wl.window_block_indices(w.seqlens, w.hkv, window)
    w_win.topk = w_win.idx.shape[2]
    c_win = Case(w_win, bwd=True, window=window)
    g_sel, g_win = wl.draw_gates(71, T, w.hq), wl.draw_gates(72, T, w.hq)
    acc_bits = wl.draw_other_branches(73, T, w.hq)
    out = dev_bf16(acc_bits).clone()
    gs, gw = torch.from_numpy(g_sel).cuda(), torch.from_numpy(g_win).cuda()
    _, o_sel, lse_sel = c_sel.attn.forward_gated(c_sel.q, c_sel.k, c_sel.v, c_sel.idx, gs, out, c_sel.cu, out=out)
    _, o_win, lse_win = c_win.attn.forward_gated(c_win.q, c_win.k, c_win.v, c_win.idx, gw, out, c_win.cu, out=out)
    torch.cuda.synchronize()
    Q, K, V, dO = c_sel.host_f64()
    r_sel, _ = orc.forward(Q, K, V, w.idx, w.cu_seqlens)
    r_win, _ = orc.forward(Q, K, V, w_win.idx, w.cu_seqlens, window=window)
    ref = orc.gated_forward(r_win, g_win.astype(np.float64),
                            orc.gated_forward(r_sel, g_sel.astype(np.float64), wl.bf16_bits_to_f64(acc_bits)))
    # three roundings to bf16 on the way (acc, + sel, + win): the absolute part of the tolerance doubles
    assert_close("out", to_f64(out), ref, (2 * TOL_O[0], TOL_O[1]))
    dq1, dk1, dv1, dg1 = c_sel.attn.backward_gated(c_sel.q, c_sel.k, c_sel.v, o_sel, lse_sel, c_sel.do, gs, c_sel.cu)
    dq2, dk2, dv2, dg2 = c_win.attn.backward_gated(c_win.q, c_win.k, c_win.v, o_win, lse_win, c_win.do, gw, c_win.cu)
    torch.cuda.synchronize()
    rq1, rk1, rv1, rg1 = orc.gated_backward(Q, K, V, dO, g_sel.astype(np.float64), w.idx, w.cu_seqlens)
    # the window branch's gradients by the same chain rule, with the window in force
    O_w, _ = orc.forward(Q, K, V, w_win.idx, w.cu_seqlens, window=window)
    rq2, rk2, rv2 = orc.backward(Q, K, V, g_win.astype(np.float64)[:, :, None] * dO, w_win.idx, w.cu_seqlens,
                                 window=window)
    rg2 = (dO * O_w).sum(axis=2)
    for name, got, want in (("dQ", dq1.float() + dq2.float(), rq1 + rq2), ("dK", dk1.float() + dk2.float(), rk1 + rk2),
                            ("dV", dv1.float() + dv2.float(), rv1 + rv2)):
        assert_close(name, to_f64(got), want, (2 * TOL_GRAD[0], TOL_GRAD[1]))
    assert_dgate_close("dgate sel", to_f64(dg1), dO, r_sel)
    assert_dgate_close("dgate win", to_f64(dg2), dO, O_w)
    assert np.allclose(rg1, (dO * r_sel).sum(axis=2)) and np.allclose(rg2, (dO * O_w).sum(axis=2))
