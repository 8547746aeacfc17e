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


def test_selection_gated_and_window_steps_replay_from_a_hip_graph():
    """The chain block scores -> selection tensor -> gated forward -> gated backward, and a sliding-window forward
    and backward on a device-made block table, recorded once and replayed on new data."""
    import paper_2508_18224_amd as nsa
    base = wl.small("g4")
    T, window = base.seqlens[0], 200
    variants = [wl.realise(dataclasses.replace(base, seed=base.seed + 100 * i)) for i in range(2)]
    scores = [torch.from_numpy(wl.draw_block_scores(500 + i, base.seqlens, base.hkv, kind="heavy")).cuda() for i in range(2)]
    gates = [torch.from_numpy(wl.draw_gates(600 + i, T, base.hq)).cuda() for i in range(2)]
    accs = [dev_bf16(wl.draw_other_branches(700 + i, T, base.hq)) for i in range(2)]

    case = Case(variants[0])
    a = case.attn
    wa = nsa.SelAttention(T, base.hq, base.hkv, -(-(window - 1) // 64) + 1, window=window)
    sc, gate, acc = scores[0].clone(), gates[0].clone(), accs[0].clone()
    idx = torch.empty(T, base.hkv, base.topk, dtype=torch.int32, device="cuda")
    widx = torch.empty(T, base.hkv, wa.shape.topk, dtype=torch.int32, device="cuda")
    import ctypes as C
    p = lambda t: C.c_void_p(t.data_ptr())
    st = lambda: C.c_void_p(torch.cuda.current_stream().cuda_stream)
    wshape = nsa.Shape(T, 1, base.hkv, base.hkv, 128, 64, wa.shape.topk, 1, 0.0, 0)

    def step():
        nsa.select_blocks(sc, case.cu, base.topk, out=idx)
        out, o, lse = a.forward_gated(case.q, case.k, case.v, idx, gate, acc, case.cu)
        g1 = a.backward_gated(case.q, case.k, case.v, o, lse, case.do, gate, case.cu)
        rc = nsa.lib().nsa_sel_select_blocks(C.byref(wshape), None, 0, p(case.cu), 0, wa.shape.topk, p(widx), st())
        assert rc == 0
        wo, wl_ = wa.forward(case.q, case.k, case.v, widx, case.cu)
        g2 = wa.backward(case.q, case.k, case.v, wo, wl_, case.do, case.cu)
        return [out, o, lse, *g1, wo, wl_, *g2]

    def load(i):
        w = variants[i]
        for dst, bits in ((case.q, w.q), (case.k, w.k), (case.v, w.v), (case.do, w.do)):
            dst.copy_(dev_bf16(bits))
        sc.copy_(scores[i]); gate.copy_(gates[i]); acc.copy_(accs[i])

    refs = []
    for i in range(2):
        load(i)
        refs.append([x.clone() for x in step()])
    torch.cuda.synchronize()
    load(0)
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        outs = step()             # tensors allocated here belong to the graph's pool and are rewritten by every replay
    for rep in (1, 0, 1):
        load(rep)
        for buf in (a.index_ws, a.fwd_ws, a.bwd_ws, wa.index_ws, wa.fwd_ws, wa.bwd_ws):
            buf.fill_(0x5A)
        _ = (case.q.float() @ case.q.float().transpose(1, 2)).sum().item()
        graph.replay()
        torch.cuda.synchronize()
        for k, (got, ref) in enumerate(zip(outs, refs[rep])):
            assert torch.equal(_bits(got), _bits(ref)), f"output {k} of replay with variant {rep} differs from eager"
