"""CPU oracle for selected-block attention (the `sel` term of the paper's Eq. (2)), forward and backward.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the HIP library is checked against; it
shares no code with the library and nothing in the product path may import it.

What is computed (paper Sec. 2.2, Eq. (2), `c = sel`; each query attends T blocks of B_K contiguous KV
tokens; causal rule from App. E: a block that is partly in the future is masked inside, a block wholly in
the future contributes nothing):

  for token t of sequence s (local position p, current block cur = p // B_K, b_s = ceil(L_s / B_K)) and KV
  head j, the selected set is  Sel = { idx[t, j, m] : 0 <= id < b_s and (not causal or id <= cur) }  (a set:
  repeated ids count once), the visible keys are the tokens u of sequence s with (u - c_s) // B_K in Sel and
  (not causal or u <= t), and for every query head h of group j (heads j*g .. j*g + g - 1; the paper prints
  floor(h / h_K), which only indexes a KV head when g = h_K, so contiguous groups are used):

      s_u = scale * <Q[t,h], K[u,j]>          LSE[t,h] = ln sum_u exp(s_u)
      p_u = exp(s_u - LSE[t,h])               O[t,h]   = sum_u p_u V[u,j]

  An empty visible set gives O = 0, LSE = -inf and no gradient.  scale defaults to 1/sqrt(d) (Eq. (1)).

Backward (the paper gives no formulas; this is the derivative of the definition above):

      delta = <dO[t,h], O[t,h]>     dp_u = <dO[t,h], V[u,j]>     ds_u = p_u (dp_u - delta)
      dQ[t,h] = scale * sum_u ds_u K[u,j]
      dK[u,j] += scale * ds_u Q[t,h]          dV[u,j] += p_u dO[t,h]      (summed over all (t,h) that see u)

Sliding window (the `win` term of Eq. (2); the paper gives neither a window length nor a kernel for it): with
window = w > 0 (causal only) a key u is visible to token t only if t - w < u <= t; run with idx listing the blocks
the window touches (the token's own block and the ceil((w - 1) / B_K) before it) the definitions above give softmax
attention over the last w tokens.  A selected block that lies wholly before the window is dropped like a future one.

Index inversion (paper Sec. 3.2: the per-KV-block query list I_i; here with the slot it came from):
  for every (KV head, global block) the ascending list of tokens that validly select it and the column of
  `idx` holding the first occurrence.  Global block ids number the blocks of the packed sequences
  consecutively (sequence 0's blocks, then sequence 1's, ...).

Gated combination (paper Eq. (2): the layer output is the sum over the three branches c of tau^c_t times the
branch's attention output).  With the other two branches' gated sum given as `O_acc`:

      O_out[t,h] = O_acc[t,h] + gate[t,h] * O[t,h]
  backward:  dO[t,h] = gate[t,h] * dO_out[t,h]  (then the backward above)     dgate[t,h] = <dO_out[t,h], O[t,h]>

  (the paper writes one gate per token and branch; a [token, head] array covers that and per-head gates alike).

All arithmetic is float64 on inputs that are bf16 values widened exactly.  No tiling, no online softmax.
Pins (tests/test_oracle_*.py): dense attention under the equivalent mask, torch's scaled_dot_product_attention
when every block is selected, torch autograd of a dense masked formulation, central finite differences, and
the closed forms listed in the tests.  The paper prints no numeric attention output, so beyond those pins the
oracle is unpinned by the paper itself.
"""
from __future__ import annotations

import math
from typing import Iterable, List, Optional, Sequence, Tuple

import numpy as np


def _seq_of(cu: np.ndarray, t: int) -> int:
    return int(np.searchsorted(cu, t, side="right") - 1)


def selected_set(idx_row: Sequence[int], cur: int, b_s: int, causal: bool, *, window: int = 0, p: int = 0,
                 block: int = 64) -> List[int]:
    """Valid block ids of one (token, kv head) row, ascending, each once.  With a window (see visible_keys) a block
    whose last token lies before the window of the token at local position p is dropped like a future block."""
    out = set()
    for x in idx_row:
        x = int(x)
        if x < 0 or x >= b_s:
            continue
        if causal and x > cur:
            continue
        if window > 0 and x != cur and (x + 1) * block - 1 < p - window + 1:
            continue
        out.add(x)
    return sorted(out)


def visible_keys(cu: np.ndarray, t: int, idx_row: Sequence[int], block: int, causal: bool,
                 window: int = 0) -> np.ndarray:
    """Global token ids of the keys token t may attend to for one kv head, ascending.  window > 0 (causal only)
    additionally hides the keys u <= t - window: with idx listing the blocks the window touches this is the
    sliding-window term of Eq. (2), softmax over the last `window` tokens."""
    assert window == 0 or causal
    s = _seq_of(cu, t)
    c0, c1 = int(cu[s]), int(cu[s + 1])
    p = t - c0
    b_s = -(-(c1 - c0) // block)
    keys: List[int] = []
    for x in selected_set(idx_row, p // block, b_s, causal, window=window, p=p, block=block):
        lo = c0 + x * block
        hi = min(lo + block, c1)
        for u in range(lo, hi):
            if causal and u > t:
                break
            if window > 0 and u <= t - window:
                continue
            keys.append(u)
    return np.asarray(keys, dtype=np.int64)


def _row_forward(q: np.ndarray, Kv: np.ndarray, Vv: np.ndarray, scale: float):
    s = scale * (Kv @ q)
    m = s.max()
    e = np.exp(s - m)
    l = e.sum()
    lse = m + math.log(l)
    p = e / l
    return p, lse, p @ Vv


def forward(Q: np.ndarray, K: np.ndarray, V: np.ndarray, idx: np.ndarray, cu: np.ndarray, *, block: int = 64,
            causal: bool = True, scale: Optional[float] = None, tokens: Optional[Iterable[int]] = None,
            window: int = 0):
    """O [T, hq, d] and LSE [T, hq] (float64).  With `tokens`, only those rows are computed (others stay 0 /
    -inf) so that a sample of a large problem can be checked."""
    T, hq, d = Q.shape
    hkv = K.shape[1]
    g = hq // hkv
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    O = np.zeros((T, hq, d), dtype=np.float64)
    LSE = np.full((T, hq), -np.inf, dtype=np.float64)
    for t in (range(T) if tokens is None else tokens):
        for j in range(hkv):
            keys = visible_keys(cu, t, idx[t, j], block, causal, window)
            if keys.size == 0:
                continue
            Kv = K[keys, j]
            Vv = V[keys, j]
            for h in range(j * g, (j + 1) * g):
                _, LSE[t, h], O[t, h] = _row_forward(Q[t, h], Kv, Vv, scale)
    return O, LSE


def backward(Q: np.ndarray, K: np.ndarray, V: np.ndarray, dO: np.ndarray, idx: np.ndarray, cu: np.ndarray, *,
             block: int = 64, causal: bool = True, scale: Optional[float] = None,
             tokens: Optional[Iterable[int]] = None, window: int = 0):
    """dQ [T, hq, d], dK, dV [T, hkv, d] (float64).  With `tokens`, only those query rows contribute (dQ of
    those rows is complete; dK/dV are then partial sums and only useful for additivity checks)."""
    T, hq, d = Q.shape
    hkv = K.shape[1]
    g = hq // hkv
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    dQ = np.zeros(Q.shape, dtype=np.float64)
    dK = np.zeros(K.shape, dtype=np.float64)
    dV = np.zeros(V.shape, dtype=np.float64)
    for t in (range(T) if tokens is None else tokens):
        for j in range(hkv):
            keys = visible_keys(cu, t, idx[t, j], block, causal, window)
            if keys.size == 0:
                continue
            Kv = K[keys, j]
            Vv = V[keys, j]
            for h in range(j * g, (j + 1) * g):
                p, _, o = _row_forward(Q[t, h], Kv, Vv, scale)
                delta = float(dO[t, h] @ o)
                dp = Vv @ dO[t, h]
                ds = p * (dp - delta)
                dQ[t, h] = scale * (ds @ Kv)
                dK[keys, j] += scale * np.outer(ds, Q[t, h])      # keys are distinct within a row
                dV[keys, j] += np.outer(p, dO[t, h])
    return dQ, dK, dV


def invert_index(idx: np.ndarray, cu: np.ndarray, *, block: int = 64, causal: bool = True,
                 kv_heads: Optional[Iterable[int]] = None, window: int = 0):
    """Per-(kv head, global block) query lists, built by one sequential pass in token order.

    Returns (cnt [hkv, b_tot] int32, off [hkv*b_tot + 1] int64 row-major over (kv head, block),
    qlist int32, qslot int32, vmask [T, hkv] uint32 with bit m set when column m of the row is a kept
    selection).  With `kv_heads`, other heads are left empty.
    """
    T, hkv, k = idx.shape
    nseq = len(cu) - 1
    nblk = [-(-(int(cu[s + 1]) - int(cu[s])) // block) for s in range(nseq)]
    base = np.concatenate([[0], np.cumsum(nblk)]).astype(np.int64)
    b_tot = int(base[-1])
    lists: List[List[Tuple[int, int]]] = [[] for _ in range(hkv * b_tot)]
    vmask = np.zeros((T, hkv), dtype=np.uint32)
    heads = range(hkv) if kv_heads is None else list(kv_heads)
    for t in range(T):
        s = _seq_of(cu, t)
        cur = (t - int(cu[s])) // block
        for j in heads:
            seen = set()
            bits = 0
            for m in range(k):
                x = int(idx[t, j, m])
                if x < 0 or x >= nblk[s] or (causal and x > cur) or x in seen:
                    continue
                if not selected_set([x], cur, nblk[s], causal, window=window, p=t - int(cu[s]), block=block):
                    continue                            # wholly before the token's window
                seen.add(x)
                bits |= 1 << m
                lists[j * b_tot + int(base[s]) + x].append((t, m))
            vmask[t, j] = bits
    cnt = np.array([len(l) for l in lists], dtype=np.int32).reshape(hkv, b_tot)
    off = np.concatenate([[0], np.cumsum(cnt.reshape(-1), dtype=np.int64)])
    flat = [e for l in lists for e in l]
    qlist = np.array([e[0] for e in flat], dtype=np.int32)
    qslot = np.array([e[1] for e in flat], dtype=np.int32)
    return cnt, off, qlist, qslot, vmask


def backward_kv_blocks(Q: np.ndarray, K: np.ndarray, V: np.ndarray, dO: np.ndarray, idx: np.ndarray,
                       cu: np.ndarray, blocks: Sequence[Tuple[int, int, int]], *, block: int = 64,
                       causal: bool = True, scale: Optional[float] = None, window: int = 0,
                       token_range: Optional[Tuple[int, int]] = None):
    """dK, dV of a few KV blocks of a large problem: `blocks` holds (kv head j, sequence s, local block x).
    Every token of sequence s that validly selects the block is revisited in full (its softmax needs all of
    its visible keys).  Returns a list of (dK_blk, dV_blk) float64 arrays of shape [keys_in_block, d].
    With `token_range` = (lo, hi) only the query tokens lo <= t < hi contribute: the sums are additive over tokens,
    so disjoint ranges can be computed side by side and added (same terms, grouped by range)."""
    T, hq, d = Q.shape
    hkv = K.shape[1]
    g = hq // hkv
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    out = []
    for (j, s, x) in blocks:
        c0, c1 = int(cu[s]), int(cu[s + 1])
        b_s = -(-(c1 - c0) // block)
        lo = c0 + x * block
        hi = min(lo + block, c1)
        dKb = np.zeros((hi - lo, d), dtype=np.float64)
        dVb = np.zeros((hi - lo, d), dtype=np.float64)
        first = lo if causal else c0
        last = c1
        if token_range is not None:
            first, last = max(first, int(token_range[0])), min(last, int(token_range[1]))
        for t in range(first, last):
            if x not in selected_set(idx[t, j], (t - c0) // block, b_s, causal, window=window, p=t - c0, block=block):
                continue
            keys = visible_keys(cu, t, idx[t, j], block, causal, window)
            inblk = (keys >= lo) & (keys < hi)
            Kv = K[keys, j]
            Vv = V[keys, j]
            for h in range(j * g, (j + 1) * g):
                p, _, o = _row_forward(Q[t, h], Kv, Vv, scale)
                delta = float(dO[t, h] @ o)
                dp = Vv @ dO[t, h]
                ds = p * (dp - delta)
                rows = keys[inblk] - lo
                dKb[rows] += scale * np.outer(ds[inblk], Q[t, h])
                dVb[rows] += np.outer(p[inblk], dO[t, h])
        out.append((dKb, dVb))
    return out


def gated_forward(O: np.ndarray, gate: np.ndarray, O_acc: Optional[np.ndarray] = None) -> np.ndarray:
    """Eq. (2) with the `sel` output O [T, hq, d], its gate [T, hq] and the other branches' gated sum O_acc."""
    out = gate[:, :, None] * O
    return out if O_acc is None else O_acc + out


def gated_backward(Q: np.ndarray, K: np.ndarray, V: np.ndarray, dO_out: np.ndarray, gate: np.ndarray, idx: np.ndarray,
                   cu: np.ndarray, *, block: int = 64, causal: bool = True, scale=None, tokens=None):
    """Gradients of a loss through O_out = O_acc + gate * O: (dQ, dK, dV, dgate).  dO_acc is dO_out itself."""
    O, _ = forward(Q, K, V, idx, cu, block=block, causal=causal, scale=scale, tokens=tokens)
    dQ, dK, dV = backward(Q, K, V, gate[:, :, None] * dO_out, idx, cu, block=block, causal=causal, scale=scale,
                          tokens=tokens)
    dgate = (dO_out * O).sum(axis=2)
    return dQ, dK, dV, dgate
