"""nsa_sel_fwd_static, the forward for callers that cannot allocate (its partial buffers live in a device array of the
library), gives the results of nsa_sel_fwd bit for bit: two calls in a row, the second on a smaller input, so that
rows the first call left in the array lie beyond and between the second call's."""
import pytest
import torch

import paper_2508_18224_amd as nsa
import workloads as wl
from gpu_util import Case

pytestmark = pytest.mark.gpu


def _both(w, window=0):
    c = Case(w, bwd=False, window=window)
    o_ref, lse_ref = c.forward()
    # poison the outputs so that a call that writes nothing cannot pass
    o = torch.full_like(o_ref, float("nan"))
    lse = torch.full_like(lse_ref, float("nan"))
    c.attn.index_ws.zero_()                                   # the static call rebuilds the index itself
    c.attn.forward_static(c.q, c.k, c.v, c.idx, c.cu, out=o, lse=lse)
    torch.cuda.synchronize()
    assert torch.equal(o.view(torch.int16), o_ref.view(torch.int16)), w.name
    assert torch.equal(lse.view(torch.int32), lse_ref.view(torch.int32)), w.name
    return c


def test_static_forward_equals_workspace_forward_on_two_calls_in_a_row():
    print("case no-alloc: large then small", flush=True)
    # 3000 tokens x 2 KV heads x g = 4 x top-k 16: one KV head's partial rows (50 MB) fit the 64 MiB array, both
    # heads' do not, so this call also runs as two passes over the same array
    big = wl.realise(wl.Workload("static_big", [1700, 1300], hq=8, hkv=2, topk=16, sink=True, seed=71))
    small = wl.realise(wl.Workload("static_small", [700], hq=8, hkv=2, topk=16, sink=True, seed=72))
    _both(big)
    _both(small)
    # other paths through the same entry point: 128-token blocks, a window, g = 7, a packed batch with an empty row set
    _both(wl.realise(wl.small("b128_g4")))
    _both(wl.realise(wl.small("g7")), window=100)
    _both(wl.realise(wl.small("g1_varlen")))


def test_static_forward_rejects_shapes_beyond_its_array():
    print("case no-alloc: too large", flush=True)
    w = wl.realise(wl.Workload("static_huge", [4200], hq=4, hkv=1, topk=16, sink=True, seed=73))
    c = Case(w, bwd=False)
    with pytest.raises(nsa.NsaSelError, match="nsa_sel_fwd_static"):
        c.attn.forward_static(c.q, c.k, c.v, c.idx, c.cu)
    o, _ = c.forward()                                         # the ordinary entry point takes the same shape
    assert bool(torch.isfinite(o.float()).all())
