"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

The oracle cannot run these shapes whole, so each case checks (a) sampled query rows (O, LSE, dQ) and sampled KV
blocks (dK, dV; every token that selects the block is revisited by the oracle) element by element, and (b)
properties that hold at any size: LSE of zero queries is the log of an exactly countable number of visible
keys, and the column sums of dV equal the summed dO of each head group (softmax rows sum to one)."""
import math

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import nsa_sel_oracle as orc
from gpu_util import BitsF64, Case, TOL_GRAD, TOL_O, TOL_LSE, assert_close, to_f64

pytestmark = pytest.mark.gpu


def _visible_counts(w):
    """Number of visible keys per (token, kv head) from the drop and mask rules, vectorised (integers)."""
    idx, cu = w.idx.astype(np.int64), w.cu_seqlens.astype(np.int64)
    T = idx.shape[0]
    tok = np.arange(T)
    seq = np.searchsorted(cu, tok, side="right") - 1
    p = tok - cu[seq]
    B = w.block
    cur = p // B
    length = cu[seq + 1] - cu[seq]
    nblk = -(-length // B)
    ok = (idx >= 0) & (idx < nblk[:, None, None]) & (idx <= cur[:, None, None])
    k = idx.shape[2]
    for m in range(1, k):                                    # first occurrence only
        ok[:, :, m] &= ~((idx[:, :, :m] == idx[:, :, m:m + 1]) & ok[:, :, :m]).any(axis=2)
    full = (ok & (idx < cur[:, None, None])).sum(axis=2) * B
    diag = (ok & (idx == cur[:, None, None])).any(axis=2) * (p % B + 1)[:, None]
    return full + diag


def _run_case(name, n_tokens, blocks, window=0):
    print("full-size case", name, "window", window, flush=True)
    w = wl.realise(wl.named(name))
    if window:                                               # the sliding-window branch at the same shape
        w.idx = wl.window_block_indices(w.seqlens, w.hkv, window, w.block)
        w.topk = w.idx.shape[2]
    T, g = w.total_tokens, w.g
    c = Case(w, window=window)
    o, lse = c.forward()
    dq, dk, dv = c.backward(o, lse)
    print("  gpu done", flush=True)
    Q, K, V, dO = (BitsF64(x) for x in (w.q, w.k, w.v, w.do))
    rng = np.random.default_rng(99)
    tokens = sorted({0, 63, 64, T - 1, *[int(x) for x in rng.integers(0, T, n_tokens)]})
    O_ref, LSE_ref = orc.forward(Q, K, V, w.idx, w.cu_seqlens, block=w.block, tokens=tokens, window=window)
    dQ_ref, _, _ = orc.backward(Q, K, V, dO, w.idx, w.cu_seqlens, block=w.block, tokens=tokens, window=window)
    sel = torch.tensor(tokens, device="cuda")
    assert_close("O", to_f64(o[sel]), O_ref[tokens], TOL_O)
    assert np.abs(to_f64(lse[sel]) - LSE_ref[tokens]).max() <= TOL_LSE
    assert_close("dQ", to_f64(dq[sel]), dQ_ref[tokens], TOL_GRAD)
    print("  sampled rows ok", flush=True)
    ref = orc.backward_kv_blocks(Q, K, V, dO, w.idx, w.cu_seqlens, blocks, block=w.block, window=window)
    for (j, s, x), (dKb, dVb) in zip(blocks, ref):
        lo = int(w.cu_seqlens[s]) + x * w.block
        hi = lo + dKb.shape[0]
        assert_close(f"dK block {(j, s, x)}", to_f64(dk[lo:hi, j]), dKb, TOL_GRAD)
        assert_close(f"dV block {(j, s, x)}", to_f64(dv[lo:hi, j]), dVb, TOL_GRAD)
    print("  sampled kv blocks ok", flush=True)
    # softmax rows sum to one: sum_u dV[u, j, :] == sum over tokens and the group's heads of dO
    want = c.do.double().view(T, w.hkv, g, 128).sum(dim=(0, 2))
    got = dv.double().sum(dim=0)
    scale_ref = c.do.double().abs().view(T, w.hkv, g, 128).sum(dim=(0, 2))
    assert float(((got - want).abs() / scale_ref).max()) < 2e-3       # bf16 rounding of dV, relative to sum |dO|
    # zero queries: LSE = ln(#visible keys), an integer count
    c.q.zero_()
    _, lse0 = c.forward(rebuild=False)
    if window:                                               # the last `window` tokens of the sequence so far
        tok = np.arange(T)
        seq = np.searchsorted(w.cu_seqlens, tok, side="right") - 1
        cnt = np.minimum(tok - w.cu_seqlens[seq] + 1, window)[:, None].repeat(w.hkv, axis=1)
    else:
        cnt = _visible_counts(w)
    want0 = torch.from_numpy(np.log(np.repeat(cnt, g, axis=1).astype(np.float64))).cuda()
    assert float((lse0.double() - want0).abs().max()) < 1e-4
    print("  closed forms ok", flush=True)


def test_headline_64k_g4():
    _run_case("headline", 12, [(0, 0, 0), (3, 0, 517), (7, 0, 1023)])


def test_headline_shape_sliding_window_512():
    _run_case("headline", 10, [(0, 0, 0), (4, 0, 600), (7, 0, 1023)], window=512)


def test_llama8b_32k_g4():
    _run_case("llama8b_32k", 8, [(2, 0, 100), (5, 0, 511)])


def test_headline_128_token_blocks():
    _run_case("headline_b128", 8, [(1, 0, 300), (6, 0, 511)])


def test_qwen_g7_64k():
    _run_case("qwen_g7", 8, [(1, 0, 300), (3, 0, 1000)])


def test_varlen_g1():
    w = wl.named("varlen_g1")
    last = len(w.seqlens) - 1
    _run_case("varlen_g1", 8, [(5, 2, 10), (15, last, 3)])


def test_llama70b_128k_g8():
    _run_case("llama70b_128k", 6, [(2, 0, 1500), (7, 0, 2047)])
