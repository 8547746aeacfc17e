"""The query-outer forward (the loop order of the original NSA kernel, kept as comparison and dispatch target) computes
the same O and LSE as the oracle, with the same drop rules, without index or workspaces."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import nsa_sel_oracle as orc
from gpu_util import Case, TOL_O, assert_close, assert_lse_close, to_f64

pytestmark = pytest.mark.gpu


def _check(w):
    c = Case(w, bwd=False)
    o, lse = c.attn.forward_query_outer(c.q, c.k, c.v, c.idx, c.cu)
    torch.cuda.synchronize()
    Q, K, V, _ = c.host_f64()
    rO, rL = orc.forward(Q, K, V, w.idx, w.cu_seqlens, causal=w.causal, block=64)
    assert_close("O", to_f64(o), rO, TOL_O)
    assert_lse_close(to_f64(lse), rL)
    return c, o, lse


@pytest.mark.parametrize("name", ["tiny", "g4", "g7", "g1_varlen", "g8", "g2_noncausal", "g4_k32", "g3_k1", "g2_hkv5"])
def test_query_outer_matches_oracle(name):
    print("case query-outer", name, flush=True)
    _check(wl.realise(wl.small(name) if name != "tiny" else wl.named("tiny")))


def test_query_outer_drop_rules_and_agreement_with_the_kv_outer_path():
    print("case query-outer adversarial", flush=True)
    w = wl.realise(wl.Workload("adv", [900, 300, 0, 65], hq=6, hkv=2, topk=10, seed=23))
    w.idx = wl.draw_adversarial_indices(np.random.default_rng(4), w.seqlens, w.hkv, w.topk)
    w.idx[100:140] = -1
    c, o, lse = _check(w)
    o2, lse2 = c.forward()
    assert not to_f64(o)[100:140].any() and np.isneginf(to_f64(lse)[100:140]).all()
    assert float((o.float() - o2.float()).abs().max()) < 2e-2 and float((lse - lse2)[torch.isfinite(lse2)].abs().max()) < 1e-3


def test_query_outer_rejects_what_it_does_not_cover():
    print("case query-outer errors", flush=True)
    import paper_2508_18224_amd as nsa
    w = wl.realise(wl.small("b128_g4"))
    c = Case(w, bwd=False)
    with pytest.raises(nsa.NsaSelError):
        c.attn.forward_query_outer(c.q, c.k, c.v, c.idx, c.cu)          # 128-token blocks
    w = wl.realise(wl.small("g4"))
    c = Case(w, bwd=False, window=100)
    with pytest.raises(nsa.NsaSelError):
        c.attn.forward_query_outer(c.q, c.k, c.v, c.idx, c.cu)          # window
