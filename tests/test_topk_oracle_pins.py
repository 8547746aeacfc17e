"""Pins of the block-selection oracle (scores -> selection tensor).  The paper does not state the selection rule
(it belongs to the cited NSA method), so the oracle is pinned to what the mathematics fixes: library sorting
routines in the special cases that reduce to them, an independent single-sort formulation, closed forms and
brute-force optimality.  The last test plants mistakes in the oracle and requires that the pins catch each."""
import math

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import topk_select_oracle as tko


def _cu(seqlens):
    return np.concatenate([[0], np.cumsum(seqlens)]).astype(np.int32)


def test_plain_topk_is_stable_argsort():
    """No forced blocks, no mask: every row is numpy's stable descending argsort cut to topk; with quantised scores
    most decisions are ties, which the stable sort resolves to the smaller block id."""
    for kind in ("heavy", "ties"):
        seqlens = [1000]
        x = wl.draw_block_scores(21, seqlens, 2, kind=kind, trap_future=False)
        got = tko.select_blocks(x, _cu(seqlens), 5, causal=False, n_sink=0, n_local=0)
        ref = np.argsort(-x.astype(np.float64), axis=2, kind="stable")[:, :, :5]
        assert np.array_equal(got, ref.astype(np.int32))


def test_selected_values_are_torch_topk_values():
    """Causal, no forced blocks: the scores of the selected blocks are torch.topk's values of the visible prefix."""
    seqlens = [900, 300]
    cu = _cu(seqlens)
    x = wl.draw_block_scores(22, seqlens, 3, kind="heavy")
    got = tko.select_blocks(x, cu, 4, causal=True, n_sink=0, n_local=0)
    for t in range(0, 1200, 37):
        s = 0 if t < 900 else 1
        cur = (t - int(cu[s])) // 64
        for j in range(3):
            k = min(4, cur + 1)
            ref = torch.topk(torch.from_numpy(x[t, j, :cur + 1]), k).values.numpy()
            sel = got[t, j]
            assert (sel[k:] == -1).all() and (sel[:k] >= 0).all()
            assert np.array_equal(x[t, j, sel[:k]], ref)


def _single_sort_row(row, cur, b_s, topk, causal, n_sink, n_local):
    """Independent route: one lexicographic sort over (class, -score, id) of all blocks, where class 0 holds the
    sinks in id order, class 1 the local blocks most recent first, class 2 the free visible ones and class 3 what
    the token cannot see."""
    b_vis = min(cur + 1, b_s) if causal else b_s
    ids = np.arange(len(row))
    cls = np.where(ids < b_vis, 2, 3)
    key = np.where(np.isnan(row), -np.inf, row.astype(np.float64))
    key = -key
    local = (ids <= cur) & (ids > cur - n_local) & (ids < b_vis)
    cls = np.where(local, 1, cls)
    key = np.where(local, (cur - ids).astype(np.float64), key)
    sink = (ids < n_sink) & (ids < b_vis)
    cls = np.where(sink, 0, cls)
    key = np.where(sink, ids.astype(np.float64), key)
    order = np.lexsort((ids, key, cls))
    order = order[cls[order] < 3][:topk]
    out = np.full(topk, -1, dtype=np.int32)
    out[:len(order)] = order
    return out


@pytest.mark.parametrize("causal,n_sink,n_local,topk,kind", [
    (True, 1, 2, 16, "heavy"), (True, 1, 2, 8, "ties"), (True, 2, 3, 6, "wild"), (False, 1, 1, 7, "wild"),
    (True, 0, 1, 1, "heavy"), (True, 3, 3, 4, "ties"), (False, 0, 0, 32, "heavy")])
def test_equals_single_lexicographic_sort(causal, n_sink, n_local, topk, kind):
    seqlens = [1100, 64, 1, 333, 129]
    cu = _cu(seqlens)
    x = wl.draw_block_scores(23, seqlens, 2, kind=kind, trap_future=causal)
    got = tko.select_blocks(x, cu, topk, causal=causal, n_sink=n_sink, n_local=n_local)
    for s, L in enumerate(seqlens):
        b_s = -(-L // 64)
        for t in range(int(cu[s]), int(cu[s + 1])):
            cur = (t - int(cu[s])) // 64
            for j in range(2):
                ref = _single_sort_row(x[t, j], cur, b_s, topk, causal, n_sink, n_local)
                assert np.array_equal(got[t, j], ref), (t, j)


def test_closed_forms():
    """Scores that rise with the block id select the most recent blocks, scores that fall select the oldest."""
    seqlens = [64 * 12]
    cu = _cu(seqlens)
    up = np.broadcast_to(np.arange(12, dtype=np.float32), (768, 1, 12)).copy()
    got = tko.select_blocks(up, cu, 5, causal=True, n_sink=1, n_local=2)
    assert got[64 * 10 + 3, 0].tolist() == [0, 10, 9, 8, 7]
    assert got[64 * 1, 0].tolist() == [0, 1, -1, -1, -1]
    assert got[5, 0].tolist() == [0, -1, -1, -1, -1]
    got = tko.select_blocks(-up, cu, 5, causal=True, n_sink=1, n_local=2)
    assert got[64 * 10 + 3, 0].tolist() == [0, 10, 9, 1, 2]
    got = tko.select_blocks(-up, cu, 5, causal=False, n_sink=0, n_local=1)
    assert got[64 * 3, 0].tolist() == [3, 0, 1, 2, 4]
    got = tko.select_blocks(np.zeros_like(up), cu, 4, causal=True, n_sink=1, n_local=1)      # all equal: smallest ids
    assert got[64 * 9, 0].tolist() == [0, 9, 1, 2]
    got = tko.select_blocks(up, cu, 2, causal=True, n_sink=2, n_local=2)                      # forced list is cut
    assert got[64 * 9, 0].tolist() == [0, 1]
    assert tko.forced_blocks(1, 2, 2, 3) == [0, 1]                                            # overlap counted once


def test_invariants_and_optimality():
    seqlens = [700, 500]
    cu = _cu(seqlens)
    x = wl.draw_block_scores(24, seqlens, 2, kind="wild")
    topk, n_sink, n_local = 6, 1, 2
    got = tko.select_blocks(x, cu, topk, causal=True, n_sink=n_sink, n_local=n_local)
    for s in range(2):
        for t in range(int(cu[s]), int(cu[s + 1])):
            cur = (t - int(cu[s])) // 64
            for j in range(2):
                row = got[t, j]
                n = min(topk, cur + 1)
                sel = row[:n]
                assert (row[n:] == -1).all()
                assert len(set(sel.tolist())) == n and sel.min() >= 0 and sel.max() <= cur
                forced = tko.forced_blocks(cur, cur + 1, n_sink, n_local)
                assert sel[:len(forced)].tolist() == forced[:n]
                val = np.where(np.isnan(x[t, j, :cur + 1]), -np.inf, x[t, j, :cur + 1])
                free = sel[len(forced):]
                rest = [b for b in range(cur + 1) if b not in sel]
                if len(free) and rest:
                    assert val[free].min() >= val[rest].max()
                assert all(val[free[i]] >= val[free[i + 1]] for i in range(len(free) - 1))


def test_nan_counts_as_minus_infinity():
    seqlens = [640]
    x = wl.draw_block_scores(25, seqlens, 1, kind="wild", trap_future=False)
    y = np.where(np.isnan(x), -np.inf, x).astype(np.float32)
    a = tko.select_blocks(x, _cu(seqlens), 9, causal=False, n_sink=0, n_local=0)
    b = tko.select_blocks(y, _cu(seqlens), 9, causal=False, n_sink=0, n_local=0)
    assert np.isnan(x).any() and np.array_equal(a, b)


# ------------------------------------------------------------------ the pins must be able to fail
def _pins():
    yield test_plain_topk_is_stable_argsort
    yield test_selected_values_are_torch_topk_values
    yield lambda: test_equals_single_lexicographic_sort(True, 1, 2, 8, "ties")
    yield lambda: test_equals_single_lexicographic_sort(False, 1, 1, 7, "wild")
    yield test_closed_forms
    yield test_invariants_and_optimality
    yield test_nan_counts_as_minus_infinity


def _some_pin_fails():
    for pin in _pins():
        try:
            pin()
        except (AssertionError, ValueError, IndexError):
            return True
    return False


def _mutant(kind):
    def select_blocks(scores, cu, topk, *, block=64, causal=True, n_sink=1, n_local=2):
        T, hkv, _ = scores.shape
        out = np.full((T, hkv, topk), -1, dtype=np.int32)
        for s in range(len(cu) - 1):
            c0, c1 = int(cu[s]), int(cu[s + 1])
            b_s = -(-(c1 - c0) // block)
            for t in range(c0, c1):
                cur = (t - c0) // block
                b_vis = (min(cur, b_s) if kind == "drops_own_block" else min(cur + 1, b_s)) if causal else b_s
                forced = tko.forced_blocks(cur, b_vis, n_sink, n_local)
                if kind == "local_before_sink":
                    forced = sorted(forced, reverse=True)
                forced = forced[:topk]
                for j in range(hkv):
                    row = scores[t, j]
                    free = [b for b in range(b_vis) if b not in forced]

                    def rank(b):
                        x = float(row[b])
                        if math.isnan(x):
                            return (-math.inf if kind == "nan_first" else math.inf, b)
                        if kind == "ascending":
                            return (x, b)
                        if kind == "ties_to_larger_id":
                            return (-x, -b)
                        return (-x, b)
                    free.sort(key=rank)
                    sel = forced + free[:topk - len(forced)]
                    if kind == "forced_not_excluded":
                        sel = forced + sorted(range(b_vis), key=rank)[:topk - len(forced)]
                    out[t, j, :len(sel)] = sel
        return out
    return select_blocks


@pytest.mark.parametrize("kind", ["ascending", "ties_to_larger_id", "drops_own_block", "local_before_sink",
                                  "nan_first", "forced_not_excluded"])
def test_planted_mistakes_are_caught(kind, monkeypatch):
    assert not _some_pin_fails()
    monkeypatch.setattr(tko, "select_blocks", _mutant(kind))
    assert _some_pin_fails(), f"no pin noticed the planted mistake '{kind}'"
