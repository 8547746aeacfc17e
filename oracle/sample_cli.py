"""Runs the CPU oracle on a sample of a named workload over several host cores and stores the results.

TEST INFRASTRUCTURE ONLY (see nsa_sel_oracle.py): used by the full-size GPU parity tests and by the cpu_baseline leg
of bench.py, as a separate process that never touches the GPU.  No arithmetic lives here: the sample is cut into
token ranges, each range is handed to nsa_sel_oracle.forward / backward / backward_kv_blocks as they stand in a
forked worker, and the per-range results are put side by side (rows of O, LSE, dQ) or added (dK/dV of a block are
sums over query tokens).  Inputs are regenerated from the workload's seed by workloads.py.

  python -m oracle.sample_cli --workload headline --tokens 0,63,64 --blocks 0:0:0,3:0:517 --out ref.npz
"""
from __future__ import annotations

import argparse
import json
import multiprocessing as mp
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import workloads as wl  # noqa: E402
from oracle import nsa_sel_oracle as orc  # noqa: E402

_G = {}  # inputs of the forked workers


class _Lazy:
    """bf16 bit patterns widened (exactly) to float64 only where indexed; optionally times a per-row factor (the
    gate folded into dO: the oracle's gated backward is its plain backward on gate * dO_out)."""

    def __init__(self, bits, row_factor=None):
        self.bits, self.row_factor = bits, row_factor
        self.shape, self.dtype = bits.shape, np.dtype(np.float64)

    def __getitem__(self, ix):
        x = wl.bf16_bits_to_f64(np.asarray(self.bits[ix]))
        if self.row_factor is not None:
            assert isinstance(ix, tuple) and len(ix) == 2          # the oracle reads dO one (token, head) row at a time
            x = x * float(self.row_factor[ix])
        return x


def _rows(tokens):
    g = _G
    kw = dict(block=g["block"], causal=g["causal"], window=g["window"])
    O, LSE = orc.forward(g["Q"], g["K"], g["V"], g["idx"], g["cu"], tokens=tokens, **kw)
    out = [O[tokens], LSE[tokens]]
    if g["bwd"]:
        dQ, _, _ = orc.backward(g["Q"], g["K"], g["V"], g["dO"], g["idx"], g["cu"], tokens=tokens, **kw)
        out.append(dQ[tokens])
    return out


def _block_part(job):
    blk, t_lo, t_hi = job
    g = _G
    (dKb, dVb), = orc.backward_kv_blocks(g["Q"], g["K"], g["V"], g["dO"], g["idx"], g["cu"], [blk], block=g["block"],
                                        causal=g["causal"], window=g["window"], token_range=(t_lo, t_hi))
    return dKb, dVb


def load(args):
    w = wl.named(args.workload) if not args.small else wl.small(args.workload)
    wl.realise(w)
    if args.window:          # the sliding-window branch at the same shape: idx = the blocks the window touches
        w.idx = wl.window_block_indices(w.seqlens, w.hkv, args.window, w.block)
        w.topk = w.idx.shape[2]
    gate = wl.draw_gates(w.seed, w.total_tokens, w.hq).astype(np.float64) if args.gated else None
    _G.update(Q=_Lazy(w.q), K=_Lazy(w.k), V=_Lazy(w.v), dO=_Lazy(w.do, gate), idx=w.idx, cu=w.cu_seqlens,
              block=w.block, causal=w.causal, window=args.window, bwd=not args.forward_only)
    return w


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", required=True)
    ap.add_argument("--small", action="store_true", help="name refers to workloads.small")
    ap.add_argument("--tokens", default="", help="comma-separated query tokens, or 'even:N' for N evenly spaced ones")
    ap.add_argument("--blocks", default="", help="comma-separated kvhead:sequence:block triples")
    ap.add_argument("--window", type=int, default=0)
    ap.add_argument("--gated", action="store_true", help="dO = gate * dO_out with workloads.draw_gates")
    ap.add_argument("--forward-only", action="store_true")
    ap.add_argument("--procs", type=int, default=0, help="worker processes (0: all host cores, at most 16)")
    ap.add_argument("--out", required=True)
    args = ap.parse_args(argv)
    procs = args.procs or min(16, len(os.sched_getaffinity(0)))
    w = load(args)
    T = w.total_tokens
    if args.tokens.startswith("even:"):
        tokens = [int(x) for x in np.linspace(0, T - 1, int(args.tokens[5:])).astype(np.int64)]
    else:
        tokens = [int(x) for x in args.tokens.split(",") if x]
    blocks = [tuple(int(y) for y in b.split(":")) for b in args.blocks.split(",") if b]
    os.environ.setdefault("OMP_NUM_THREADS", "1")
    try:
        from threadpoolctl import threadpool_limits
        limiter = threadpool_limits(limits=1)        # one BLAS thread per worker: the workers are the parallelism
    except ImportError:                              # pragma: no cover
        limiter = None
    res = {"tokens": np.asarray(tokens, dtype=np.int64), "procs": np.int64(procs)}
    ctx = mp.get_context("fork")
    with ctx.Pool(procs) as pool:
        t0 = time.perf_counter()
        if tokens:
            chunks = [c.tolist() for c in np.array_split(np.asarray(tokens), min(len(tokens), 4 * procs)) if len(c)]
            parts = pool.map(_rows, chunks, chunksize=1)
            res["O"] = np.concatenate([p[0] for p in parts])
            res["LSE"] = np.concatenate([p[1] for p in parts])
            if not args.forward_only:
                res["dQ"] = np.concatenate([p[2] for p in parts])
        res["rows_seconds"] = np.float64(time.perf_counter() - t0)
        t0 = time.perf_counter()
        for n, blk in enumerate(blocks):
            j, s, x = blk
            c0, c1 = int(w.cu_seqlens[s]), int(w.cu_seqlens[s + 1])
            first = c0 + x * w.block if w.causal else c0
            edges = np.linspace(first, c1, min(4 * procs, max(1, (c1 - first) // 64)) + 1).astype(np.int64)
            jobs = [(blk, int(a), int(b)) for a, b in zip(edges[:-1], edges[1:]) if b > a]
            parts = pool.map(_block_part, jobs, chunksize=1)
            res[f"dK{n}"] = sum(p[0] for p in parts)
            res[f"dV{n}"] = sum(p[1] for p in parts)
        res["blocks_seconds"] = np.float64(time.perf_counter() - t0)
    del limiter
    np.savez(args.out, **res)
    print(json.dumps({"tokens": len(tokens), "blocks": len(blocks), "procs": procs,
                      "rows_seconds": float(res["rows_seconds"]), "blocks_seconds": float(res["blocks_seconds"])}),
          flush=True)


if __name__ == "__main__":
    main()
