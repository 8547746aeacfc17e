"""Seeded synthetic inputs for selected-block attention (shared by the oracle tests and the HIP tests).

This module holds no attention arithmetic: it only draws tensors and block-index tables.  Both the CPU
oracle and the HIP library are fed from here so that they see bit-identical bf16 inputs.

Shapes follow the paper's kernel grid (d = 128, B_K = 64, T = 16, Llama/Qwen head counts; Sec. 4.1 and
the appendix on ultra-long sequence lengths).  The paper does not say how its selection indices were
drawn, so each workload states its own recipe: forced blocks (attention sink = block 0, App. E, the paragraph on
the attention sink; the current block; optionally the previous block), a number of picks biased to the most
recent blocks, and the rest uniform without replacement over the remaining earlier blocks.  Rows are left in
generation order (forced, local, uniform) and padded with -1.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

BLOCK = 64
HEAD_DIM = 128


# ----------------------------------------------------------------------------- bf16 plumbing
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns the 16-bit patterns as uint16."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns exactly to float32."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns exactly to float64."""
    return bf16_bits_to_f32(bits).astype(np.float64)


# ----------------------------------------------------------------------------- workload description
@dataclass
class Workload:
    name: str
    seqlens: List[int]
    hq: int
    hkv: int
    topk: int
    causal: bool = True
    sink: bool = False            # block 0 forced into every row
    recent: int = 1               # number of forced most-recent blocks (1 = current block only)
    local_picks: int = 0          # picks drawn from the `local_window` blocks before the forced recent ones
    local_window: int = 8
    seed: int = 0
    d: int = HEAD_DIM
    block: int = BLOCK
    # filled by realise()
    cu_seqlens: Optional[np.ndarray] = None
    idx: Optional[np.ndarray] = None
    q: Optional[np.ndarray] = None
    k: Optional[np.ndarray] = None
    v: Optional[np.ndarray] = None
    do: Optional[np.ndarray] = None
    extra: dict = field(default_factory=dict)

    @property
    def total_tokens(self) -> int:
        return int(sum(self.seqlens))

    @property
    def g(self) -> int:
        return self.hq // self.hkv


def _floyd_subsets(rng: np.random.Generator, n: np.ndarray, m: int) -> np.ndarray:
    """Uniform random subsets without replacement, one per row (Floyd's algorithm, vectorised over rows).

    Row r receives min(m, n[r]) distinct integers from [0, n[r]); unused columns hold -1.
    """
    rows = n.shape[0]
    out = np.full((rows, max(m, 1)), -1, dtype=np.int64)
    if m == 0:
        return out[:, :0]
    n = n.astype(np.int64)
    take = np.minimum(n, m)
    for i in range(m):
        active = i < take
        jmax = n - take + i                      # candidate range is [0, jmax]
        u = rng.random(rows)
        r = np.minimum((u * (jmax + 1)).astype(np.int64), jmax)
        if i > 0:
            clash = (out[:, :i] == r[:, None]).any(axis=1)
            r = np.where(clash, jmax, r)
        out[:, i] = np.where(active, r, -1)
    return out


def draw_block_indices(rng: np.random.Generator, seqlens: Sequence[int], hkv: int, topk: int, *, sink: bool,
                       recent: int, local_picks: int, local_window: int, block: int = BLOCK) -> np.ndarray:
    """int32 [total_tokens, hkv, topk] of sequence-local block ids, -1 padded; selections independent per
    (token, kv head)."""
    per_seq = []
    for L in seqlens:
        cur = (np.arange(L, dtype=np.int64) // block)                      # current block of each token
        cur = np.repeat(cur[:, None], hkv, axis=1).reshape(-1)              # rows = (token, kv head)
        rows = cur.shape[0]
        cols = []
        if sink:
            cols.append(np.zeros(rows, dtype=np.int64))
        for r in range(recent):
            c = cur - r
            c = np.where(c >= 0, c, -1)
            if sink:
                c = np.where(c == 0, -1, c)                                 # already forced as the sink
            cols.append(c)
        lo = 1 if sink else 0
        hi = np.maximum(cur - (recent - 1), lo)                            # earlier pool is [lo, hi)
        n_forced = len(cols)
        n_free = topk - n_forced
        assert n_free >= 0
        n_local = min(local_picks, n_free)
        n_unif = n_free - n_local
        if n_local > 0:
            llo = np.maximum(hi - local_window, lo)
            picks = _floyd_subsets(rng, hi - llo, n_local)
            cols.extend(list(np.where(picks >= 0, picks + llo[:, None], -1).T))
            uhi = llo
        else:
            uhi = hi
        if n_unif > 0:
            picks = _floyd_subsets(rng, uhi - lo, n_unif)
            cols.extend(list(np.where(picks >= 0, picks + lo, -1).T))
        table = np.stack(cols, axis=1)                                      # [rows, topk]
        # compact the valid ids to the front, keeping generation order; pad the tail with -1
        order = np.argsort(table < 0, axis=1, kind="stable")
        table = np.take_along_axis(table, order, axis=1)
        per_seq.append(table.reshape(L, hkv, topk))
    return np.concatenate(per_seq, axis=0).astype(np.int32)


def realise(w: Workload, *, tensors: bool = True) -> Workload:
    """Draw the index table and (optionally) the bf16 Q/K/V/dO tensors of a workload from its seed."""
    rng = np.random.default_rng(w.seed)
    T = w.total_tokens
    w.cu_seqlens = np.concatenate([[0], np.cumsum(w.seqlens)]).astype(np.int32)
    w.idx = draw_block_indices(rng, w.seqlens, w.hkv, w.topk, sink=w.sink, recent=w.recent,
                               local_picks=w.local_picks, local_window=w.local_window, block=w.block)
    if tensors:
        w.q = _draw_bf16(w.seed, 0, T, w.hq, w.d)
        w.k = _draw_bf16(w.seed, 1, T, w.hkv, w.d)
        w.v = _draw_bf16(w.seed, 2, T, w.hkv, w.d)
        w.do = _draw_bf16(w.seed, 3, T, w.hq, w.d)
    return w


_SLAB_TOKENS = 2048


def _draw_bf16(seed: int, tensor: int, T: int, heads: int, d: int) -> np.ndarray:
    """Standard-normal values rounded to bf16, [T, heads, d] as bit patterns.  Every slab of 2048 tokens has
    its own generator seeded by (seed, tensor, slab), so the result does not depend on how many threads draw."""
    out = np.empty((T, heads, d), dtype=np.uint16)

    def work(t0: int):
        t1 = min(t0 + _SLAB_TOKENS, T)
        r = np.random.default_rng([seed, tensor, t0 // _SLAB_TOKENS])
        out[t0:t1] = f32_to_bf16_bits(r.standard_normal((t1 - t0, heads, d), dtype=np.float32))

    with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as pool:
        list(pool.map(work, range(0, T, _SLAB_TOKENS)))
    return out


# ----------------------------------------------------------------------------- named workloads
def varlen_lengths(seed: int, nseq: int = 8, lo: int = 4096, hi: int = 32768) -> List[int]:
    rng = np.random.default_rng(seed)
    return [int(x) for x in rng.integers(lo, hi + 1, size=nseq)]


def named(name: str) -> Workload:
    """The benchmark configurations: 'tiny', 'llama8b_32k', 'headline', 'qwen_g7', 'varlen_g1', 'llama70b_128k'."""
    if name == "tiny":            # config 1
        return Workload(name, [1024], hq=4, hkv=1, topk=8, seed=1001)
    if name == "llama8b_32k":     # config 2
        return Workload(name, [32768], hq=32, hkv=8, topk=16, sink=True, seed=1002)
    if name == "headline":        # the metric's shape: config 2's heads at N = 64k, g = 4
        return Workload(name, [65536], hq=32, hkv=8, topk=16, sink=True, seed=1000)
    if name == "qwen_g7":         # config 3
        return Workload(name, [65536], hq=28, hkv=4, topk=16, sink=True, local_picks=7, local_window=8,
                        seed=1003)
    if name == "varlen_g1":       # config 4
        return Workload(name, varlen_lengths(1004), hq=16, hkv=16, topk=16, seed=1004)
    if name == "llama70b_128k":   # config 5
        return Workload(name, [131072], hq=64, hkv=8, topk=16, sink=True, recent=2, seed=1005)
    if name == "headline_b128":   # the headline shape at the paper's second setting (B_K, T) = (128, 8)
        return Workload(name, [65536], hq=32, hkv=8, topk=8, sink=True, block=128, seed=1006)
    if name.startswith("grid_"):
        # the paper's kernel grid (Sec. 4.1): grid_g<g>_b<B_K>_n<N in K>[_h<query heads>], 32 query heads unless
        # given (the 128K / 256K tables of App. F use 64)
        parts = dict((p[0], int(p[1:])) for p in name.split("_")[1:])
        g, block, n, hq = parts["g"], parts["b"], parts["n"] * 1024, parts.get("h", 32)
        return Workload(name, [n], hq=hq, hkv=hq // g, topk=1024 // block, sink=True, block=block,
                        seed=2000 + 100 * g + block + parts["n"] + (hq if hq != 32 else 0))
    raise KeyError(name)


NAMES = ["tiny", "llama8b_32k", "headline", "qwen_g7", "varlen_g1", "llama70b_128k"]


def small(name: str) -> Workload:
    """Scaled-down cases for element-wise parity: same recipes, sizes the oracle finishes in seconds.
    Lengths are not multiples of 64 so that tiles have ragged tails."""
    if name == "g4":
        return Workload(name, [2000], hq=8, hkv=2, topk=16, sink=True, seed=11)
    if name == "g7":
        return Workload(name, [1500], hq=7, hkv=1, topk=16, sink=True, local_picks=7, seed=12)
    if name == "g1_varlen":
        return Workload(name, [700, 64, 1, 333, 1029], hq=3, hkv=3, topk=16, seed=13)
    if name == "g8":
        return Workload(name, [1800], hq=8, hkv=1, topk=16, sink=True, recent=2, seed=14)
    if name == "g2_noncausal":
        return Workload(name, [900, 450], hq=4, hkv=2, topk=8, causal=False, seed=15)
    if name == "g4_k32":
        return Workload(name, [2500], hq=4, hkv=1, topk=32, sink=True, seed=16)
    if name == "g3_k1":
        return Workload(name, [777], hq=3, hkv=1, topk=1, seed=17)
    if name == "g2_hkv5":       # several KV heads, a sink list long enough to split into work units
        return Workload(name, [2300, 700], hq=10, hkv=5, topk=8, sink=True, seed=20)
    if name == "b128_g4":       # the paper's second setting (B_K, T) = (128, 8)
        return Workload(name, [2100], hq=8, hkv=2, topk=8, sink=True, block=128, seed=18)
    if name == "b128_varlen":
        return Workload(name, [700, 129, 128, 1, 515], hq=2, hkv=2, topk=4, block=128, seed=19)
    raise KeyError(name)


SMALL_NAMES = ["g4", "g7", "g1_varlen", "g8", "g2_noncausal", "g4_k32", "g3_k1", "g2_hkv5", "b128_g4", "b128_varlen"]


def draw_adversarial_indices(rng: np.random.Generator, seqlens: Sequence[int], hkv: int, topk: int,
                             block: int = BLOCK) -> np.ndarray:
    """Index rows that exercise the drop rules: ids anywhere in [-2, b_s + 2) (future blocks, out-of-range
    ids, padding in the middle of a row) with repeats."""
    per_seq = []
    for L in seqlens:
        b = -(-L // block)
        tab = rng.integers(-2, b + 2, size=(L, hkv, topk))
        dup = rng.random((L, hkv, topk)) < 0.25
        tab = np.where(dup, np.roll(tab, 1, axis=2), tab)
        per_seq.append(tab)
    return np.concatenate(per_seq, axis=0).astype(np.int32)


# ----------------------------------------------------------------------------- block scores (input of the selection step)
def draw_block_scores(seed: int, seqlens: Sequence[int], hkv: int, block: int = BLOCK, *, kind: str = "heavy",
                      stride: Optional[int] = None, trap_future: bool = True) -> np.ndarray:
    """float32 [total_tokens, hkv, stride] block-importance scores, stride >= blocks of the longest sequence.

    The paper publishes no score data; the recipe imitates what the compression branch of NSA hands over
    (attention mass per block, summed over the heads of a group): positive, heavy-tailed, with more mass on
    recent blocks.
      'heavy'  exp(1.5 z) * (1 + 2 exp(-(cur - b) / 8)), z standard normal
      'ties'   the same, quantised to 8 levels, so that most comparisons are ties
      'wild'   standard normal with a sprinkle of +-inf, NaN, +-0 and denormals
    With trap_future the columns of blocks after the token's own block hold huge values: a causal selection must
    never read them.  Every slab of 2048 tokens has its own generator, like the bf16 tensors."""
    T = int(sum(seqlens))
    nb = max(-(-int(L) // block) for L in seqlens)
    stride = nb if stride is None else stride
    assert stride >= nb
    cu = np.concatenate([[0], np.cumsum(seqlens)]).astype(np.int64)
    out = np.empty((T, hkv, stride), dtype=np.float32)
    cols = np.arange(stride, dtype=np.int64)

    def work(t0: int):
        t1 = min(t0 + _SLAB_TOKENS, T)
        r = np.random.default_rng([seed, 7, t0 // _SLAB_TOKENS])
        z = r.standard_normal((t1 - t0, hkv, stride), dtype=np.float32)
        tok = np.arange(t0, t1, dtype=np.int64)
        s = np.searchsorted(cu, tok, side="right") - 1
        cur = ((tok - cu[s]) // block)[:, None, None]
        if kind in ("heavy", "ties"):
            age = np.maximum(cur - cols[None, None, :], 0).astype(np.float32)
            x = np.exp(np.float32(1.5) * z) * (1 + 2 * np.exp(-age / np.float32(8)))
            if kind == "ties":
                x = np.floor(np.minimum(x, 7.0))
        elif kind == "wild":
            x = z.copy()
            u = r.random((t1 - t0, hkv, stride))
            for lo, val in ((0.00, np.inf), (0.03, -np.inf), (0.06, np.nan), (0.09, 0.0), (0.12, -0.0),
                            (0.15, 1e-42), (0.18, -1e-42)):
                x[(u >= lo) & (u < lo + 0.03)] = val
        else:
            raise KeyError(kind)
        if trap_future:
            x = np.where(cols[None, None, :] > cur, np.float32(3e38), x)
        out[t0:t1] = x.astype(np.float32)

    with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as pool:
        list(pool.map(work, range(0, T, _SLAB_TOKENS)))
    return out


# ----------------------------------------------------------------------------- gates (input of the gated combination)
def draw_gates(seed: int, T: int, hq: int) -> np.ndarray:
    """float32 [T, hq] gate values in [0, 1]: a logistic squashing of standard normals (what a sigmoid gate layer
    emits), with about 2 % of the entries set to exactly 0 and 2 % to exactly 1."""
    r = np.random.default_rng([seed, 8])
    g = (1.0 / (1.0 + np.exp(-1.5 * r.standard_normal((T, hq))))).astype(np.float32)
    u = r.random((T, hq))
    g[u < 0.02] = 0.0
    g[u > 0.98] = 1.0
    return g


def draw_other_branches(seed: int, T: int, hq: int, d: int = HEAD_DIM) -> np.ndarray:
    """bf16 bit patterns [T, hq, d]: a stand-in for the gated sum of the other attention branches."""
    return _draw_bf16(seed, 4, T, hq, d)


# ----------------------------------------------------------------------------- sliding-window rows
def window_block_indices(seqlens: Sequence[int], hkv: int, window: int, block: int = BLOCK) -> np.ndarray:
    """int32 [total_tokens, hkv, R + 1], R = ceil((window - 1) / block): the token's own block and the R blocks before
    it, most recent first, -1 where the sequence has no such block.  These are the blocks a causal window of
    `window` tokens can touch; which of their keys are inside the window is decided by whoever consumes the table."""
    R = -(-(window - 1) // block)
    per_seq = []
    for L in seqlens:
        cur = np.arange(L, dtype=np.int64) // block
        tab = cur[:, None] - np.arange(R + 1, dtype=np.int64)[None, :]
        tab = np.where(tab >= 0, tab, -1)
        per_seq.append(np.repeat(tab[:, None, :], hkv, axis=1))
    return np.concatenate(per_seq, axis=0).astype(np.int32)
