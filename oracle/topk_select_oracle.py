"""CPU oracle for the step in front of the selected-attention path: block scores -> selection tensor.

TEST INFRASTRUCTURE ONLY.  Slow, plain definition the HIP library's selection kernel is checked against; it
shares no code with the library and nothing in the product path may import it.

What is computed.  The paper takes the selection tensor (Sec. 2.2: every query token of a GQA group attends to
its own T KV blocks of B_K tokens) as given and only notes that block 0, the attention sink, ends up selected by
every token (App. E, the paragraph on the attention sink).  How the T blocks are chosen belongs to the cited NSA
method and is not stated in the paper: PARITY UNPINNED by the paper.  The rule implemented here, and pinned in
tests/test_topk_oracle_pins.py to library sorting routines, brute force and closed forms, is

  for token t of sequence s (local position p, own block cur = p // B_K, b_s = ceil(L_s / B_K) blocks) and KV
  head j, with scores[t, j, b] the importance of block b of the token's sequence:

    visible   = { b : 0 <= b < b_s and (not causal or b <= cur) }
    forced    = the first n_sink blocks (0, 1, ...) and then the token's n_local most recent blocks
                (cur, cur - 1, ...), each once, in that order, as far as they are visible
    free      = the visible blocks that are not forced, ordered by descending score, equal scores by
                ascending block id; a NaN score counts as -infinity
    idx[t, j] = forced, then the first topk - |forced| free blocks, then -1 padding        (length topk)

  (if topk is smaller than the number of forced blocks, the forced list is cut to its first topk entries).
  Comparisons are made on the fp32 values as given: no arithmetic is applied to a score.
"""
from __future__ import annotations

import math

import numpy as np


def forced_blocks(cur: int, b_vis: int, n_sink: int, n_local: int):
    """Blocks every row selects regardless of score: sinks first, then most recent first; ids < b_vis, each once."""
    out = []
    for b in range(n_sink):
        if b < b_vis and b not in out:
            out.append(b)
    for r in range(n_local):
        b = cur - r
        if 0 <= b < b_vis and b not in out:
            out.append(b)
    return out


def select_blocks(scores: np.ndarray, cu: np.ndarray, topk: int, *, block: int = 64, causal: bool = True,
                  n_sink: int = 1, n_local: int = 2, tokens=None) -> np.ndarray:
    """scores: float32 [total_tokens, hkv, >= max blocks per sequence]; returns int32 [total_tokens, hkv, topk].
    With `tokens` only those rows are computed (the others stay -1)."""
    T, hkv, _ = scores.shape
    out = np.full((T, hkv, topk), -1, dtype=np.int32)
    wanted = None if tokens is None else set(int(t) for t in tokens)
    for s in range(len(cu) - 1):
        c0, c1 = int(cu[s]), int(cu[s + 1])
        b_s = -(-(c1 - c0) // block)
        for t in (range(c0, c1) if wanted is None else sorted(x for x in wanted if c0 <= x < c1)):
            cur = (t - c0) // block
            b_vis = min(cur + 1, b_s) if causal else b_s
            forced = forced_blocks(cur, b_vis, n_sink, n_local)[:topk]
            for j in range(hkv):
                row = scores[t, j]
                free = [b for b in range(b_vis) if b not in forced]

                def rank(b):
                    x = float(row[b])
                    return (math.inf if math.isnan(x) else -x, b)      # descending score, ascending block id
                free.sort(key=rank)
                sel = forced + free[:topk - len(forced)]
                out[t, j, :len(sel)] = sel
    return out
