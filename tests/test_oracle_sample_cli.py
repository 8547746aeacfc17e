"""The multi-process sampling front end of the oracle (oracle/sample_cli.py) adds no arithmetic: its rows equal those
of nsa_sel_oracle.forward / backward called directly, and its per-block dK/dV (summed over token ranges) equal
backward_kv_blocks in one piece up to the order of the additions."""
import numpy as np

import workloads as wl
from oracle import nsa_sel_oracle as orc
from oracle import sample_cli


def _direct(name, window=0, gated=False):
    w = wl.realise(wl.small(name))
    if window:
        w.idx = wl.window_block_indices(w.seqlens, w.hkv, window, w.block)
    Q, K, V, dO = (wl.bf16_bits_to_f64(x) for x in (w.q, w.k, w.v, w.do))
    if gated:
        dO = wl.draw_gates(w.seed, w.total_tokens, w.hq).astype(np.float64)[:, :, None] * dO
    return w, Q, K, V, dO


def test_sampled_rows_and_blocks_equal_the_direct_oracle(tmp_path):
    for name, window, gated in (("g4", 0, False), ("g1_varlen", 130, False), ("b128_g4", 0, True)):
        w, Q, K, V, dO = _direct(name, window, gated)
        T = w.total_tokens
        tokens = [0, 1, 63, 64, 65, T // 2, T - 1]
        blocks = [(0, 0, 0), (w.hkv - 1, len(w.seqlens) - 1, -(-w.seqlens[-1] // w.block) - 1), (0, 0, 3)]
        out = tmp_path / f"{name}.npz"
        argv = ["--workload", name, "--small", "--procs", "3", "--out", str(out), "--tokens",
                ",".join(map(str, tokens)), "--blocks", ",".join(":".join(map(str, b)) for b in blocks)]
        if window:
            argv += ["--window", str(window)]
        if gated:
            argv.append("--gated")
        sample_cli.main(argv)
        ref = np.load(out)
        kw = dict(block=w.block, causal=w.causal, window=window)
        O, LSE = orc.forward(Q, K, V, w.idx, w.cu_seqlens, tokens=tokens, **kw)
        dQ, _, _ = orc.backward(Q, K, V, dO, w.idx, w.cu_seqlens, tokens=tokens, **kw)
        assert np.array_equal(ref["O"], O[tokens]) and np.array_equal(ref["LSE"], LSE[tokens])
        assert np.array_equal(ref["dQ"], dQ[tokens])
        whole = orc.backward_kv_blocks(Q, K, V, dO, w.idx, w.cu_seqlens, blocks, **kw)
        for n, (dKb, dVb) in enumerate(whole):
            assert np.allclose(ref[f"dK{n}"], dKb, rtol=1e-12, atol=1e-12)
            assert np.allclose(ref[f"dV{n}"], dVb, rtol=1e-12, atol=1e-12)
            assert np.abs(dKb).max() > 0
