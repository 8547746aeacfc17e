"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

The oracle cannot run these shapes whole, so each case checks (a) >= 256 sampled query rows (O, LSE, dQ) and >= 8
sampled KV blocks including the last one (dK, dV; every token that selects the block is revisited by the oracle)
element by element - at the headline, the varlen and the 128-token-block shapes also a block whose query list is split
over several work units, which exercises the fixed-order dK/dV reduction - and (b) properties that hold at any size:
LSE of zero queries is the log of an exactly countable number of visible keys, and the column sums of dV equal the
summed dO of each head group (softmax rows sum to one).

The oracle runs as a separate process (oracle/sample_cli.py: nsa_sel_oracle as it stands, token ranges spread over
the host's cores) that regenerates the same seeded inputs and never touches the GPU; it is started before the GPU
work of the case and joined afterwards."""
import os
import subprocess
import sys
import tempfile

import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import Case, TOL_GRAD, TOL_O, TOL_LSE, assert_close, assert_dgate_close, dev_bf16, to_f64

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


class OracleRun:
    """The oracle on `tokens` / `blocks` of a named workload, in a child process."""

    def __init__(self, name, tokens, blocks, window=0, gated=False, forward_only=False):
        self.tokens, self.blocks = list(tokens), list(blocks)
        self.path = tempfile.mktemp(suffix=".npz", prefix="nsa_ref_")
        cmd = [sys.executable, "-m", "oracle.sample_cli", "--workload", name, "--out", self.path,
               "--tokens", ",".join(str(t) for t in self.tokens),
               "--blocks", ",".join(":".join(str(x) for x in b) for b in self.blocks)]
        if window:
            cmd += ["--window", str(window)]
        if gated:
            cmd.append("--gated")
        if forward_only:
            cmd.append("--forward-only")
        self.proc = subprocess.Popen(cmd, cwd=ROOT, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)

    def result(self):
        out, _ = self.proc.communicate(timeout=900)
        assert self.proc.returncode == 0, out
        print("  oracle:", out.strip().splitlines()[-1], flush=True)
        ref = dict(np.load(self.path))
        os.unlink(self.path)
        assert [int(t) for t in ref["tokens"]] == self.tokens
        return ref


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


def _sample_tokens(T, n, seed=99):
    rng = np.random.default_rng(seed)
    return sorted({0, 63, 64, T - 1, *[int(x) for x in rng.integers(0, T, n)]})


def _sample_blocks(w0, n, extra=(), seed=7):
    """n (kv head, sequence, block) triples spread over heads and positions, always with the last block of the last
    sequence, plus `extra`."""
    rng = np.random.default_rng(seed)
    nseq = len(w0.seqlens)
    out = list(extra)
    last_s = nseq - 1
    out.append((w0.hkv - 1, last_s, -(-w0.seqlens[last_s] // w0.block) - 1))
    while len(out) < n + len(extra):
        s = int(rng.integers(0, nseq))
        nb = -(-w0.seqlens[s] // w0.block)
        cand = (int(rng.integers(0, w0.hkv)), s, int(rng.integers(1, nb)))
        if cand not in out:
            out.append(cand)
    return out


def _check_rows(ref, tokens, o, lse, dq):
    sel = torch.tensor(tokens, device="cuda")
    assert_close("O", to_f64(o[sel]), ref["O"], TOL_O)
    got, want = to_f64(lse[sel]), ref["LSE"]
    assert np.array_equal(np.isneginf(got), np.isneginf(want))
    fin = np.isfinite(want)
    assert np.abs(got[fin] - want[fin]).max() <= TOL_LSE
    if dq is not None:
        assert_close("dQ", to_f64(dq[sel]), ref["dQ"], TOL_GRAD)
    print(f"  {len(tokens)} sampled rows ok", flush=True)


def _check_blocks(ref, w, blocks, dk, dv):
    for n, (j, s, x) in enumerate(blocks):
        dKb, dVb = ref[f"dK{n}"], ref[f"dV{n}"]
        lo = int(w.cu_seqlens[s]) + x * w.block
        hi = lo + dKb.shape[0]
        assert_close(f"dK block {(j, s, x)}", to_f64(dk[lo:hi, j]), dKb, TOL_GRAD)
        assert_close(f"dV block {(j, s, x)}", to_f64(dv[lo:hi, j]), dVb, TOL_GRAD)
    print(f"  {len(blocks)} sampled kv blocks ok", flush=True)


def _run_case(name, n_tokens=256, n_blocks=8, extra_blocks=(), window=0, closed_forms=True, dense=None):
    """dense=None: the forward routing the library picks for the shape, i.e. what bench.py times."""
    print("full-size case", name, "window", window, "dense", dense, flush=True)
    w0 = wl.named(name)
    tokens = _sample_tokens(w0.total_tokens, n_tokens)
    blocks = _sample_blocks(w0, n_blocks, extra_blocks)
    oracle = OracleRun(name, tokens, blocks, window=window)
    w = wl.realise(wl.named(name))
    if window:                                               # the sliding-window branch at the same shape
        w.idx = wl.window_block_indices(w.seqlens, w.hkv, window, w.block)
        w.topk = w.idx.shape[2]
    T, g = w.total_tokens, w.g
    c = Case(w, window=window, dense=dense)
    o, lse = c.forward()
    dq, dk, dv = c.backward(o, lse)
    print("  gpu done; dense share of the pairs:", round(float(c.attn.dense_entries().mean()), 3), flush=True)
    if extra_blocks:                                         # these lists must really be split over work units
        cnt, _, _, _, _, _ = c.attn.index_arrays()
        for (j, s, x) in extra_blocks:
            gb = sum(-(-L // w.block) for L in w.seqlens[:s]) + x
            assert cnt[j, gb] > 2048, (j, s, x, int(cnt[j, gb]))
    ref = oracle.result()
    _check_rows(ref, tokens, o, lse, dq)
    _check_blocks(ref, w, blocks, dk, dv)
    if not closed_forms:
        return
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
    _run_case("headline", extra_blocks=[(0, 0, 0)])           # the sink block's list: 32 work units


def test_headline_shape_sliding_window_512():
    _run_case("headline", window=512)


def test_llama8b_32k_g4():
    _run_case("llama8b_32k")


def test_headline_128_token_blocks():
    _run_case("headline_b128", extra_blocks=[(5, 0, 0)])


def test_qwen_g7_64k():
    _run_case("qwen_g7")


def test_varlen_g1():
    w = wl.named("varlen_g1")
    shortest = int(np.argmin(w.seqlens))
    _run_case("varlen_g1", extra_blocks=[(9, shortest, 0)])   # first block of the shortest sequence: > 1 work unit


def test_llama70b_128k_g8():
    _run_case("llama70b_128k")


@pytest.mark.parametrize("name", ["grid_g1_b128_n64", "grid_g8_b128_n64"])
def test_128_token_blocks_at_g1_and_g8(name):
    _run_case(name, n_tokens=128, n_blocks=4, closed_forms=False)


def test_ultra_long_256k_tokens_64_heads():
    """The largest shape of the paper's grid (App. F): 256K tokens, 64 query heads (g = 8), (B_K, T) = (64, 16)."""
    _run_case("grid_g8_b64_n256_h64", n_tokens=64, n_blocks=4)


def test_headline_with_the_gather_route_only():
    """The routing the library does not pick at the headline shape (shape.dense = -1), forward rows only."""
    _run_case("headline", n_blocks=1, closed_forms=False, dense=False)


def test_varlen_g1_with_the_dense_route_forced():
    """g = 1 runs the gather route by default; the dense route at that shape (shape.dense = 1)."""
    _run_case("varlen_g1", n_blocks=1, closed_forms=False, dense=True)


def test_headline_gated_entry_points():
    """nsa_sel_fwd_gated / nsa_sel_bwd_gated at the headline shape: O_out, dQ, dgate on sampled rows, dK/dV on sampled
    blocks (the oracle's gated backward is its backward on gate * dO_out)."""
    name = "headline"
    print("full-size case gated", name, flush=True)
    w0 = wl.named(name)
    tokens = _sample_tokens(w0.total_tokens, 256, seed=5)
    blocks = _sample_blocks(w0, 4, seed=11)
    oracle = OracleRun(name, tokens, blocks, gated=True)
    w = wl.realise(wl.named(name))
    T = w.total_tokens
    c = Case(w, dense=None)
    gate = wl.draw_gates(w.seed, T, w.hq)
    acc_bits = wl.draw_other_branches(w.seed, T, w.hq)
    gate_d, acc_d = torch.from_numpy(gate).cuda(), dev_bf16(acc_bits)
    o_out, o, lse = c.attn.forward_gated(c.q, c.k, c.v, c.idx, gate_d, acc_d, c.cu)
    dq, dk, dv, dgate = c.attn.backward_gated(c.q, c.k, c.v, o, lse, c.do, gate_d, c.cu)
    torch.cuda.synchronize()
    print("  gpu done", flush=True)
    ref = oracle.result()
    _check_rows(ref, tokens, o, lse, dq)
    _check_blocks(ref, w, blocks, dk, dv)
    from oracle import nsa_sel_oracle as orc
    sel = torch.tensor(tokens, device="cuda")
    rO = ref["O"]                                            # the ungated output (the gate only scales dO)
    g64 = gate.astype(np.float64)[tokens]
    assert_close("O_out", to_f64(o_out[sel]), orc.gated_forward(rO, g64, wl.bf16_bits_to_f64(acc_bits[tokens])), TOL_O)
    assert_dgate_close("dgate", to_f64(dgate[sel]), wl.bf16_bits_to_f64(w.do[tokens]), rO)
    off = torch.from_numpy(gate == 0.0).cuda()
    assert bool(off.any()) and not bool(dq[off].any())        # a closed gate passes no gradient


def test_headline_query_outer_forward():
    """nsa_sel_fwd_query_outer at the headline shape on sampled rows."""
    name = "headline"
    print("full-size case query-outer", name, flush=True)
    w0 = wl.named(name)
    tokens = _sample_tokens(w0.total_tokens, 256, seed=3)
    oracle = OracleRun(name, tokens, [], forward_only=True)
    w = wl.realise(wl.named(name))
    c = Case(w, bwd=False)
    o, lse = c.attn.forward_query_outer(c.q, c.k, c.v, c.idx, c.cu)
    torch.cuda.synchronize()
    _check_rows(oracle.result(), tokens, o, lse, None)
