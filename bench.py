#!/usr/bin/env python3
"""Benchmark of the selected-attention hot path on one MI355X.

A step is one pass of the whole path on the headline workload (N = 65536, hq = 32, hkv = 8, g = 4, top-k 16,
block 64, d = 128, causal, seeded synthetic bf16 inputs already resident in HBM): index inversion, forward
(main + merge), backward (delta, main, dQ reduce, dK/dV reduce).  Prints ONE JSON line: effective TFLOP/s
(4 N hq k 64 d forward + 2.5x backward, per the paper's FLOP count for the selected kernel), a roofline object
for the dominant kernel, and the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0

# kernel kinds of nsa_sel_profile_collect -> kernel names in the rocprofv3 summaries under profiles/
KERNEL_NAMES = {
    "fwd_main": ("nsa::k_fwd_main", "nsa::k_fwd_main128"), "fwd_merge": ("nsa::k_fwd_merge",),
    "fwd_dense": ("nsa::k_fwd_dense_merge",),
    "bwd_main": ("nsa::k_bwd_tiled<2>", "nsa::k_bwd_pipe128"), "bwd_delta": ("nsa::k_bwd_delta",),
    "bwd_dq_reduce": ("nsa::k_bwd_dq_reduce",), "bwd_dkv_reduce": ("nsa::k_bwd_dkv_reduce",),
}
NOT_IN_STEP = ("nsa::k_select_blocks", "k_calib_copy", "nsa::k_mfma_probe", "nsa::k_fwd_query_outer")


def measured_traffic(workload: str):
    """{kernel name: HBM bytes per launch} from the committed rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary of
    this workload (profiles/hot_path_<workload>.txt, the table headed 'HBM traffic per launch', already scaled by the
    copy-kernel calibration).  The counters cannot be read inside a timing run, so the summary is the source; a
    workload without one has no traffic figure and the caller says so loudly."""
    path = os.path.join(ROOT, "profiles", f"hot_path_{workload}.txt")
    if not os.path.exists(path):
        return None, path
    out, on = {}, False
    for line in open(path):
        if line.startswith("HBM traffic per launch"):
            on = True
        elif on:
            parts = line.split()
            if len(parts) == 4 and parts[0] != "kernel":
                try:
                    out[parts[0]] = float(parts[3]) * 1e9
                except ValueError:
                    pass
    return out, path


def cpu_baseline(workload: str, budget_tokens: int):
    """The fp64 oracle, as it stands, on evenly spaced tokens of the same workload (forward, then backward), spread
    over the host's cores by oracle/sample_cli.py in a child process that never touches the GPU.  Called before this
    process initialises the GPU."""
    import subprocess
    import tempfile

    import workloads as wl
    from paper_2508_18224_amd.cost_model import effective_flops
    out = tempfile.mktemp(suffix=".npz", prefix="nsa_cpu_baseline_")
    cmd = [sys.executable, "-m", "oracle.sample_cli", "--workload", workload, "--tokens", f"even:{budget_tokens}",
           "--out", out]
    res = subprocess.run(cmd, cwd=ROOT, capture_output=True, text=True)
    if res.returncode != 0:
        sys.exit("bench.py: the CPU oracle sample failed:\n" + res.stdout + res.stderr)
    info = json.loads(res.stdout.strip().splitlines()[-1])
    os.unlink(out)
    w = wl.named(workload)
    f, b = effective_flops(info["tokens"], w.hq, w.topk, block=w.block)
    dt = info["rows_seconds"]
    return {"value": (f + b) / dt / 1e12, "unit": "TFLOP/s", "cores": info["procs"], "kind": "oracle",
            "sample": f"{info['tokens']} evenly spaced query tokens of the same workload, all heads, forward + "
                      f"backward contributions of those rows, {dt:.1f} s wall on {info['procs']} worker processes "
                      f"(one per host core)"}


def bench_select_blocks(nsa, wl, w, cu, steps):
    """The step in front of the path, measured on its own (it is not part of the metric's step): seeded fp32 block
    scores of the workload's shape -> selection tensor.  HBM-bound: every visible score is read once."""
    import torch
    nb_max = max(-(-L // w.block) for L in w.seqlens)
    if 4 * w.total_tokens * w.hkv * nb_max > 12e9:
        return {"skipped": "the score tensor of this shape exceeds 12 GB of host memory to draw"}
    t0 = time.time()
    x = torch.from_numpy(wl.draw_block_scores(w.seed, w.seqlens, w.hkv, w.block, kind="heavy")).cuda()
    print(f"[bench] block scores drawn in {time.time() - t0:.1f} s", file=sys.stderr, flush=True)
    out = torch.empty(w.total_tokens, w.hkv, w.topk, dtype=torch.int32, device="cuda")
    kw = dict(block=w.block, causal=w.causal, n_sink=1, n_local=2, out=out)
    for _ in range(3):
        nsa.select_blocks(x, cu, w.topk, **kw)
    torch.cuda.synchronize()
    nsa.profile_select(["select_blocks"])
    nsa.profile_enable(steps)
    for _ in range(steps):
        nsa.select_blocks(x, cu, w.topk, **kw)
    torch.cuda.synchronize()
    tot, n = nsa.profile_collect()["select_blocks"]
    nsa.profile_enable(0)
    nsa.profile_select(None)
    ms = tot / n
    # algorithmic bytes: the visible scores (4 B each) plus the idx rows written
    vis = 0
    for L in w.seqlens:
        nb = -(-L // w.block)
        cur = np.arange(L, dtype=np.int64) // w.block
        vis += int((cur + 1).sum()) if w.causal else L * nb
    nbytes = 4 * (vis * w.hkv + w.total_tokens * w.hkv * w.topk)
    gbs = nbytes / (ms * 1e-3) / 1e9
    return {"ms_per_launch": ms, "algorithmic_bytes": nbytes, "bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS,
            "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS, "scores": "seeded 'heavy' recipe of workloads.draw_block_scores, "
            "1 sink + 2 local blocks forced"}


def bench_extras(nsa, wl, w, q, k, v, do, cu, steps):
    """Steps after the path, measured on their own (not part of the metric): the gated forms of forward and backward
    against the plain ones, and the sliding-window branch run through the same kernels, on the workload's tensors."""
    import torch
    T = w.total_tokens

    def per_kernel(run):
        for _ in range(2):
            run()
        torch.cuda.synchronize()
        nsa.profile_select(None)
        nsa.profile_enable(steps * (24 + 8 * w.hkv))
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(steps):
            run()
        b.record()
        torch.cuda.synchronize()
        prof = nsa.profile_collect()
        nsa.profile_enable(0)
        out = {n: t / c for n, (t, c) in prof.items() if c and not n.startswith("index_")}
        out["step_with_events"] = a.elapsed_time(b) / steps
        return out

    res = {}
    idx = torch.from_numpy(w.idx).cuda()
    attn = nsa.SelAttention(T, w.hq, w.hkv, w.topk, nseq=len(w.seqlens), causal=w.causal, block=w.block)
    gate = torch.from_numpy(wl.draw_gates(w.seed, T, w.hq)).cuda()
    acc = torch.from_numpy(wl.draw_other_branches(w.seed, T, w.hq).view(np.int16)).cuda().view(torch.bfloat16)

    def plain():
        o, lse = attn.forward(q, k, v, idx, cu)
        attn.backward(q, k, v, o, lse, do, cu)

    def gated():
        _, o, lse = attn.forward_gated(q, k, v, idx, gate, acc, cu, out=acc)
        attn.backward_gated(q, k, v, o, lse, do, gate, cu)
    res["plain"] = per_kernel(plain)
    res["gated"] = per_kernel(gated)
    if w.block == 64:
        # the paper's comparison on this chip: the same forward in the original NSA (query-outer) loop order
        def kv_outer_fwd():
            attn.forward(q, k, v, idx, cu)

        def query_outer_fwd():
            attn.forward_query_outer(q, k, v, idx, cu)
        a = per_kernel(kv_outer_fwd)
        b = per_kernel(query_outer_fwd)
        res["loop_order_forward"] = {"kv_outer_ms": a["step_with_events"], "query_outer_ms": b["step_with_events"],
                                     "ratio": b["step_with_events"] / a["step_with_events"],
                                     "note": "kv_outer includes index inversion, main and merge"}
        # What a query-outer kernel that shares blocks between the tokens of a 64-token query tile could reach at
        # best: only the forced blocks (sink, own, recent) are shared by a tile's tokens, and for those the
        # query-tile-outer order is this library's dense route; the other picks differ from token to token and cost
        # a K/V block load per (token, block) in any query-outer cut.  So: the query-outer kernel on the free picks
        # alone plus the dense route on the forced blocks alone.
        tok = np.arange(T)
        seq = np.searchsorted(w.cu_seqlens, tok, side="right") - 1
        cur = ((tok - w.cu_seqlens[seq]) // w.block)[:, None, None]
        forced = np.zeros(w.idx.shape, dtype=bool)
        if w.sink:
            forced |= w.idx == 0
        for r in range(w.recent):
            forced |= w.idx == cur - r
        idx_free = torch.from_numpy(np.where(forced, -1, w.idx).astype(np.int32)).cuda()
        idx_forced = torch.from_numpy(np.where(forced, w.idx, -1).astype(np.int32)).cuda()
        dense_attn = nsa.SelAttention(T, w.hq, w.hkv, w.topk, nseq=len(w.seqlens), causal=w.causal, block=w.block,
                                      bwd=False, dense=True)
        c = per_kernel(lambda: attn.forward_query_outer(q, k, v, idx_free, cu))
        d = per_kernel(lambda: dense_attn.forward(q, k, v, idx_forced, cu))
        res["loop_order_forward"].update({
            "query_outer_free_picks_only_ms": c["step_with_events"],
            "query_tile_outer_forced_blocks_only_ms": d["step_with_events"],
            "query_outer_with_sharing_estimate_ms": c["step_with_events"] + d["step_with_events"],
            "forced_share_of_pairs": float(forced.sum()) / float((w.idx >= 0).sum())})
        del idx_free, idx_forced, dense_attn
    del attn, idx
    if w.causal:
        for window, blk in ((512, 64), (512, 128)):
            widx = nsa.window_blocks(T, w.hkv, window, cu, block=blk)
            wattn = nsa.SelAttention(T, w.hq, w.hkv, widx.shape[2], nseq=len(w.seqlens), causal=True, block=blk,
                                     window=window)

            def win():
                o, lse = wattn.forward(q, k, v, widx, cu)
                wattn.backward(q, k, v, o, lse, do, cu)
            res[f"window_{window}_block_{blk}"] = dict(per_kernel(win), slots=int(widx.shape[2]))
            del wattn, widx
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="headline")
    ap.add_argument("--calibrate", action="store_true",
                    help="also launch the library's 1 GiB copy kernel once (for scaling rocprofv3 byte counters)")
    ap.add_argument("--unit", type=int, default=0,
                    help="list entries per work unit (0: the library's choice; a power of two in 256..2048)")
    ap.add_argument("--ws-cap-gb", type=float, default=0.0,
                    help="cap each workspace at this many GB: the library then reuses it over groups of KV heads")
    ap.add_argument("--dense", choices=["auto", "on", "off"], default="auto",
                    help="routing of the forward (shape.dense): the library's choice, or the dense route forced on / off")
    ap.add_argument("--no-select", action="store_true",
                    help="skip the separate measurement of the selection step (block scores -> idx) in front of the path")
    ap.add_argument("--extras", action="store_true",
                    help="also measure the gated forms and the sliding-window branch (reported under 'downstream')")
    ap.add_argument("--cpu-tokens", type=int, default=8192, help="query tokens of the CPU-oracle sample (0: skip)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the path shards over KV heads with no "
                 "communication, so N GPUs would each run this same kernel on hkv / N heads); run with --gpus 1")

    # the CPU baseline first: its worker processes are forked before this process has touched the GPU, and the
    # host is idle again when the GPU timing starts
    cpu = cpu_baseline(args.workload, args.cpu_tokens) if args.cpu_tokens > 0 else None
    if cpu is not None:
        print(f"[bench] cpu oracle: {cpu['value']:.4f} TFLOP/s on {cpu['cores']} cores", file=sys.stderr, flush=True)

    import torch

    import paper_2508_18224_amd as nsa
    import workloads as wl
    from paper_2508_18224_amd.cost_model import compulsory_bytes, effective_flops

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    nsa.lib()  # fail loudly if the HIP library is missing
    t0 = time.time()
    w = wl.realise(wl.named(args.workload))
    print(f"[bench] inputs drawn in {time.time() - t0:.1f} s", file=sys.stderr, flush=True)
    T = w.total_tokens

    def dev(bits):
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    q, k, v, do = (dev(x) for x in (w.q, w.k, w.v, w.do))
    idx = torch.from_numpy(w.idx).cuda()
    cu = torch.from_numpy(w.cu_seqlens).cuda()
    attn = nsa.SelAttention(T, w.hq, w.hkv, w.topk, nseq=len(w.seqlens), causal=w.causal, block=w.block, unit=args.unit,
                            dense={'auto': None, 'on': True, 'off': False}[args.dense], ws_cap_bytes=int(args.ws_cap_gb * 1e9) if args.ws_cap_gb > 0 else None)
    o = torch.empty_like(q)
    lse = torch.empty(T, w.hq, dtype=torch.float32, device="cuda")
    grads = (torch.empty_like(q), torch.empty_like(k), torch.empty_like(v))

    def step():
        attn.forward(q, k, v, idx, cu, rebuild_index=True, out=o, lse=lse)
        attn.backward(q, k, v, o, lse, do, cu, out=grads)

    if args.calibrate:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").zero_()
        dst = torch.empty_like(src)
        nsa.calibration_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst
    # what this chip delivers to plain kernels of this build: a register-resident MFMA loop and a streaming copy
    def _timed(fn):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fn()
        torch.cuda.synchronize()
        a.record()
        fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e-3
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    probe_flops = nsa.mfma_probe(20000, sink)
    mfma_measured = probe_flops / _timed(lambda: nsa.mfma_probe(20000, sink)) / 1e12
    cp_src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").zero_()
    cp_dst = torch.empty_like(cp_src)
    copy_measured = 2 * (1 << 30) / _timed(lambda: nsa.calibration_copy(cp_dst, cp_src)) / 1e9
    del cp_src, cp_dst
    print(f"[bench] measured on this chip: MFMA loop {mfma_measured:.0f} TFLOP/s, streaming copy {copy_measured:.0f} GB/s",
          file=sys.stderr, flush=True)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # Untimed pass with an event pair around EVERY kernel launch: the per-kernel breakdown, and which kernel
    # dominates.  (An event pair costs a few microseconds of stream time, ~1 % of a step when all ~18 launches
    # carry one, so the timed region below records the dominant kernel only.)
    cap = 24 + 8 * w.hkv   # launches per step, also with a capped workspace
    n_prof = min(args.steps, 5)
    nsa.profile_select(None)
    nsa.profile_enable(n_prof * cap)
    for _ in range(n_prof):
        step()
    torch.cuda.synchronize()
    prof = nsa.profile_collect()
    per_kernel = {name: tot / n for name, (tot, n) in prof.items() if n}
    dom = max(per_kernel, key=per_kernel.get)
    nsa.profile_select([dom])
    nsa.profile_enable(args.steps * cap)
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        marks[i].record()      # on the launch stream, no synchronisation: per-step spread only
        step()
    marks[args.steps].record()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    live = nsa.profile_collect()   # the dominant kernel, timed with HIP events inside the timed region
    nsa.profile_enable(0)
    nsa.profile_select(None)
    per_kernel[dom] = live[dom][0] / live[dom][1]

    f, b = effective_flops(T, w.hq, w.topk, block=w.block)
    for name, avg in sorted(per_kernel.items(), key=lambda kv: -kv[1]):
        print(f"[bench] {name:16s} {avg:9.3f} ms/launch", file=sys.stderr)
    fwd_ms = sum(per_kernel.get(n, 0.0) for n in ("fwd_main", "fwd_dense", "fwd_merge"))
    bwd_ms = sum(per_kernel.get(n, 0.0) for n in ("bwd_delta", "bwd_main", "bwd_dq_reduce", "bwd_dkv_reduce"))
    idx_ms = sum(vv for n, vv in per_kernel.items() if n.startswith("index_"))
    # algorithmic work of the dominant kernel: the MFMA contractions it performs (forward main: QK^T and PV,
    # 4 N hq k 64 d; backward main: five such products, 2.5x)
    dom_flops = {"fwd_main": f, "bwd_main": b}.get(dom)
    alg_f, alg_b = compulsory_bytes(T, w.hq, w.hkv, w.topk)
    traffic, traffic_file = measured_traffic(args.workload)
    if traffic is None:
        print(f"[bench] WARNING: {traffic_file} does not exist: no rocprofv3 byte-counter summary for this workload, "
              f"roofline.traffic is null", file=sys.stderr, flush=True)
    roof = None
    if dom_flops is not None:
        sec = per_kernel[dom] * 1e-3
        ach = dom_flops / sec / 1e12
        # the compulsory bytes of the pass the kernel dominates (forward or backward), each tensor once
        alg = alg_f if dom == "fwd_main" else alg_b
        tr = None
        if traffic is not None:
            tr = next((traffic[k] for k in KERNEL_NAMES[dom] if k in traffic), None)
            if tr is None and not args.calibrate:
                sys.exit(f"bench.py: {traffic_file} has no row for {KERNEL_NAMES[dom]}: regenerate the summary")
            if tr is None:  # --calibrate is the run that regenerates the summary
                print(f"[bench] WARNING: {traffic_file} has no row for {KERNEL_NAMES[dom]}, roofline.traffic is null",
                      file=sys.stderr, flush=True)
        roof = {"kernel": dom, "bound": "mfma", "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": ach / PEAK_BF16_TFLOPS, "traffic": tr, "ms_per_launch": per_kernel[dom],
                "algorithmic_flops": dom_flops, "algorithmic_bytes": alg,
                # the same launch against the HBM roofline on ALGORITHMIC bytes (wasted traffic lowers it)
                "hbm_algorithmic": {"achieved": alg / sec / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                    "frac": alg / sec / 1e9 / PEAK_HBM_GBS},
                "traffic_ratio": None if tr is None else tr / alg,
                "traffic_source": os.path.relpath(traffic_file, ROOT) if traffic is not None else None}
    step_traffic = None
    if traffic is not None:
        step_bytes = sum(v for k, v in traffic.items() if not k.startswith(NOT_IN_STEP))
        step_traffic = {"counter_bytes_per_step": step_bytes, "algorithmic_bytes_per_step": alg_f + alg_b,
                        "traffic_ratio": step_bytes / (alg_f + alg_b),
                        "hbm_algorithmic_frac": (alg_f + alg_b) / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS}
    out = {
        "metric": "selected-attn fwd+bwd effective TFLOP/s & ms at N=64k, g=4 (frac of MFMA peak)",
        "value": (f + b) / (ms * 1e-3) / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: N={T}, hq={w.hq}, hkv={w.hkv}, g={w.g}, topk={w.topk}, block={w.block}, "
                               f"d=128, causal, seed {w.seed}",
                   "step": "index inversion + forward (main, dense, merge) + backward (delta, main, dQ reduce, dK/dV reduce)",
                   "workspace_GB": {"fwd": attn.fwd_ws.numel() / 1e9, "bwd": attn.bwd_ws.numel() / 1e9,
                                    "index": attn.index_ws.numel() / 1e9}},
        "frac_of_bf16_mfma_peak": (f + b) / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "ms": {"index": idx_ms, "fwd": fwd_ms, "bwd": bwd_ms, "per_kernel": per_kernel,
               "step_median": per_step[len(per_step) // 2], "step_min": per_step[0]},
        "roofline": roof,
        "step_traffic": step_traffic,
        "measured_peaks": {"mfma_loop_TFLOPs": mfma_measured, "stream_copy_GBps": copy_measured,
                           "frac_of_measured_mfma": (f + b) / (ms * 1e-3) / 1e12 / mfma_measured},
    }
    if not args.no_select:
        out["upstream"] = {"select_blocks": bench_select_blocks(nsa, wl, w, cu, args.steps)}
    if args.extras:
        del attn
        out["downstream"] = bench_extras(nsa, wl, w, q, k, v, do, cu, min(args.steps, 5))
    if cpu is not None:
        out["cpu_baseline"] = cpu
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
