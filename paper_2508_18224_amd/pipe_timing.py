"""Where the waves of the pipelined 128-key backward kernel spend their clocks.

    python -m paper_2508_18224_amd.pipe_timing [--workload headline_b128]

Runs one backward pass of a (B_K = 128) workload through `libnsa_sel_timing.so`, the library built from the same sources
with -DNSA_PIPE_TIMING (paper_2508_18224_amd/build.py): there k_bwd_pipe128 reads the shader clock at the four points of
every pipeline step and adds up, per role, the clocks between them.  The results of that build are the same as the
product library's; its times are a few percent higher (each stamp waits for the wave's outstanding LDS operations).
Prints one line per role: mean clocks per wave and work unit in each phase.
"""
from __future__ import annotations

import argparse
import ctypes
import os
import sys

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PHASES = ("wait at the first barrier (staged tile / P, dS ready)", "products of the step",
          "wait at the second barrier (tiles free)", "after it: staging and row request (S) / nothing (A)")


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="headline_b128")
    args = ap.parse_args()
    from paper_2508_18224_amd import binding
    from paper_2508_18224_amd.build import LIB_TIMING
    if not os.path.exists(LIB_TIMING):
        sys.exit(f"{LIB_TIMING} is missing: run `python -m paper_2508_18224_amd.build` first")
    binding._LIB_PATH = LIB_TIMING  # before the first call: the binding loads its library lazily
    import paper_2508_18224_amd as nsa
    import workloads as wl

    w = wl.realise(wl.named(args.workload))
    if w.block != 128:
        sys.exit("the pipelined kernel serves 128-token blocks: pick a (128, T) workload")

    def dev(bits):
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    q, k, v, do = (dev(x) for x in (w.q, w.k, w.v, w.do))
    idx = torch.from_numpy(w.idx).cuda()
    cu = torch.from_numpy(w.cu_seqlens).cuda()
    att = nsa.SelAttention(w.total_tokens, w.hq, w.hkv, w.topk, nseq=len(w.seqlens), causal=w.causal, block=w.block)
    o, lse = att.forward(q, k, v, idx, cu)
    for _ in range(3):
        att.backward(q, k, v, o, lse, do, cu)
    torch.cuda.synchronize()
    h = ctypes.CDLL(LIB_TIMING)
    out = (ctypes.c_ulonglong * 16)()
    if h.nsa_sel_pipe_timing_read(out, 1) != 0:
        sys.exit("reading the timers failed")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    att.backward(q, k, v, o, lse, do, cu)
    e1.record()
    torch.cuda.synchronize()
    if h.nsa_sel_pipe_timing_read(out, 1) != 0:
        sys.exit("reading the timers failed")
    t = np.array(list(out), dtype=np.float64).reshape(2, 8)
    rows = w.total_tokens * w.hq * w.topk
    print(f"workload {args.workload}: one backward pass (delta, main, both reductions) in {e0.elapsed_time(e1):.3f} ms "
          f"with the timing build; the main kernel works through {rows / 64:.0f} tiles of 64 rows x 128 keys")
    for r, name in enumerate(("P/dS waves (0-3)", "accumulating waves (4-7)")):
        n = t[r, 4]
        units = n / 4
        per_tile = t[r, :4] / n / (rows / 64 / units)
        print(f"{name}: {int(n)} waves = {int(units)} work units; mean clocks per wave and 64-row tile:")
        for ph, c in zip(PHASES, per_tile):
            print(f"    {c:8.0f}  {ph}")
        print(f"    {per_tile.sum():8.0f}  total")


if __name__ == "__main__":
    main()
