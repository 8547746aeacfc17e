"""Index inversion on the GPU must equal the oracle's sequential inversion bit for bit."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import nsa_sel_oracle as orc

pytestmark = pytest.mark.gpu


def _compare(w, idx_override=None):
    import paper_2508_18224_amd as nsa
    idx = w.idx if idx_override is None else idx_override
    attn = nsa.SelAttention(w.total_tokens, w.hq, w.hkv, w.topk, nseq=len(w.seqlens), causal=w.causal, bwd=False,
                            block=w.block)
    attn.build_index(torch.from_numpy(idx).cuda(), torch.from_numpy(w.cu_seqlens).cuda())
    torch.cuda.synchronize()
    cnt, off, qlist, qslot, vmask, bcap = attn.index_arrays()
    rc, ro, rl, rs, rv = orc.invert_index(idx, w.cu_seqlens, causal=w.causal, block=w.block)
    b_tot = rc.shape[1]
    assert bcap >= b_tot
    assert np.array_equal(cnt[:, :b_tot], rc) and not cnt[:, b_tot:].any()
    for j in range(w.hkv):
        assert np.array_equal(off[j * bcap: j * bcap + b_tot].astype(np.int64), ro[j * b_tot:(j + 1) * b_tot])
    assert int(off[-1]) == int(ro[-1])
    assert np.array_equal(qlist, rl)
    assert np.array_equal(qslot, rs)
    assert np.array_equal(vmask, rv)


@pytest.mark.parametrize("name", wl.SMALL_NAMES + ["tiny"])
def test_inversion_bit_exact(name):
    print("case", name, flush=True)
    w = wl.realise(wl.small(name) if name != "tiny" else wl.named("tiny"), tensors=False)
    _compare(w)


@pytest.mark.parametrize("causal", [True, False])
def test_inversion_drop_rules(causal):
    """Future, out-of-range, padding and repeated ids are dropped exactly as the oracle drops them."""
    print("adversarial causal", causal, flush=True)
    w = wl.Workload("adv", [1000, 77, 640], hq=4, hkv=2, topk=12, causal=causal, seed=5)
    wl.realise(w, tensors=False)
    idx = wl.draw_adversarial_indices(np.random.default_rng(8), w.seqlens, w.hkv, w.topk)
    _compare(w, idx)
    w.block = 128                                   # same rows read as ids of 128-token blocks
    _compare(w, idx)


def test_inversion_multi_chunk_scan():
    """Enough lists x chunks that the scan needs more than one level, and chunks that straddle sequences."""
    print("multi-level scan", flush=True)
    w = wl.Workload("big", [5000, 3000, 4100], hq=4, hkv=4, topk=16, sink=True, seed=6)
    wl.realise(w, tensors=False)
    _compare(w)


@pytest.mark.parametrize("name,heads", [("headline", [0, 5]), ("varlen_g1", [3]), ("llama70b_128k", [7])])
def test_inversion_bit_exact_full_size(name, heads):
    """Benchmark-size tables; the oracle's sequential pass is run for a few kv heads only (it is per-head)."""
    import paper_2508_18224_amd as nsa
    print("full-size inversion", name, flush=True)
    w = wl.realise(wl.named(name), tensors=False)
    attn = nsa.SelAttention(w.total_tokens, w.hq, w.hkv, w.topk, nseq=len(w.seqlens), causal=True, bwd=False)
    attn.build_index(torch.from_numpy(w.idx).cuda(), torch.from_numpy(w.cu_seqlens).cuda())
    torch.cuda.synchronize()
    cnt, off, qlist, qslot, vmask, bcap = attn.index_arrays()
    rc, ro, rl, rs, rv = orc.invert_index(w.idx, w.cu_seqlens, kv_heads=heads)
    b_tot = rc.shape[1]
    for j in heads:
        assert np.array_equal(cnt[j, :b_tot], rc[j]) and not cnt[j, b_tot:].any()
        lo, hi = int(off[j * bcap]), int(off[j * bcap + b_tot])
        rlo, rhi = int(ro[j * b_tot]), int(ro[(j + 1) * b_tot])
        assert hi - lo == rhi - rlo
        assert np.array_equal(qlist[lo:hi], rl[rlo:rhi])
        assert np.array_equal(qslot[lo:hi], rs[rlo:rhi])
        assert np.array_equal(vmask[:, j], rv[:, j])
    # sink pattern: block 0 of every head is selected by every token (App. E, attention sink)
    if w.sink:
        assert np.all(cnt[:, 0] == w.total_tokens)
    assert int(off[-1]) == int(cnt.sum())
