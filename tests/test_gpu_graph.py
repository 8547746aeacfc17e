"""The library neither allocates nor synchronises, so a whole step (index inversion + forward + backward) can
be recorded into a HIP graph.  The graph is replayed several times, with eager work, poisoned workspaces and
NEW input data (same shape, other seed) between the replays; every replay must reproduce the eager results
bit for bit."""
import dataclasses

import pytest
import torch

import workloads as wl
from gpu_util import Case, dev_bf16

pytestmark = pytest.mark.gpu


def _eager(w):
    case = Case(w)
    o, lse = case.forward()
    dq, dk, dv = case.backward(o, lse)
    return [x.clone() for x in (o, lse, dq, dk, dv)]


def _bits(x):
    return x.view(torch.int16) if x.dtype == torch.bfloat16 else x.view(torch.int32)


@pytest.mark.parametrize("name", ["g4", "b128_g4"])
def test_step_replays_from_a_hip_graph(name):
    base = wl.small(name)
    variants = [wl.realise(dataclasses.replace(base, seed=base.seed + 100 * i)) for i in range(3)]
    refs = [_eager(w) for w in variants]

    case = Case(variants[0])      # static buffers the graph is recorded on
    a = case.attn
    o = torch.empty_like(case.q)
    lse = torch.empty(case.w.total_tokens, case.w.hq, dtype=torch.float32, device="cuda")
    grads = (torch.empty_like(case.q), torch.empty_like(case.k), torch.empty_like(case.v))

    def step():
        a.forward(case.q, case.k, case.v, case.idx, case.cu, rebuild_index=True, out=o, lse=lse)
        a.backward(case.q, case.k, case.v, o, lse, case.do, case.cu, out=grads)

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        step()                    # first launches outside the capture (kernel attributes are set here)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()

    for rep in (1, 2, 0, 1):
        w = variants[rep]
        for dst, bits in ((case.q, w.q), (case.k, w.k), (case.v, w.v), (case.do, w.do)):
            dst.copy_(dev_bf16(bits))
        case.idx.copy_(torch.from_numpy(w.idx).cuda())
        for buf in (a.index_ws, a.fwd_ws, a.bwd_ws):
            buf.fill_(0x5A)       # nothing may survive from the previous replay
        for t in (o, lse, *grads):
            t.zero_()
        _ = (case.q.float() @ case.q.float().transpose(1, 2)).sum().item()   # unrelated eager work + sync
        graph.replay()
        torch.cuda.synchronize()
        for nm, got, ref in zip(("O", "LSE", "dQ", "dK", "dV"), (o, lse, *grads), refs[rep]):
            assert torch.equal(_bits(got), _bits(ref)), f"{nm} of replay with variant {rep} differs from eager"
