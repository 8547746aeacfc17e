"""The pins must be able to fail: each plausible mistake planted in the oracle (on the CPU, by patching it) has to
trip at least one of the pin tests."""
import math

import numpy as np
import pytest

import test_oracle_pins as pins
from oracle import nsa_sel_oracle as orc


def _pins():
    case = pins.CASES[1]
    yield lambda: pins.test_forward_equals_dense_masked_attention(case)
    yield lambda: pins.test_backward_equals_autograd_of_dense_masked_attention(case)
    yield lambda: pins.test_forward_equals_dense_masked_attention(pins.CASES[3])
    yield lambda: pins.test_all_blocks_selected_is_full_attention(True)
    yield pins.test_backward_matches_central_finite_differences
    yield pins.test_closed_forms
    yield lambda: pins.test_inversion_against_mask_and_invariants(pins.CASES[4])


def _some_pin_fails():
    for pin in _pins():
        try:
            pin()
        except (AssertionError, ValueError, IndexError):
            return True
    return False


def _row_forward_no_scale(q, Kv, Vv, scale):
    return orc_row_forward(q, Kv, Vv, 1.0)


def _visible_keys_no_inblock_mask(cu, t, idx_row, block, causal, window=0):
    s = orc._seq_of(cu, t)
    c0, c1 = int(cu[s]), int(cu[s + 1])
    keys = []
    for x in orc.selected_set(idx_row, (t - c0) // block, -(-(c1 - c0) // block), causal):
        keys.extend(range(c0 + x * block, min(c0 + (x + 1) * block, c1)))        # forgets u <= t
    return np.asarray(keys, dtype=np.int64)


def _selected_set_drops_current(idx_row, cur, b_s, causal, **kw):
    return sorted({int(x) for x in idx_row if 0 <= int(x) < b_s and (not causal or int(x) < cur)})   # < for <=


def _selected_set_multiset(idx_row, cur, b_s, causal, **kw):
    return sorted(int(x) for x in idx_row if 0 <= int(x) < b_s and (not causal or int(x) <= cur))   # repeats kept


orc_row_forward = orc._row_forward
orc_backward = orc.backward


def _backward_mutated(kind):
    def backward(Q, K, V, dO, idx, cu, *, block=64, causal=True, scale=None, tokens=None):
        dQ, dK, dV = orc_backward(Q, K, V, dO, idx, cu, block=block, causal=causal, scale=scale, tokens=tokens)
        sc = 1.0 / math.sqrt(Q.shape[2]) if scale is None else scale
        if kind == "dk_unscaled":
            dK = dK / sc
        elif kind == "dq_sign":
            dQ = -dQ
        elif kind == "dv_one_head":                      # sums one head of the group instead of all g
            g = Q.shape[1] // K.shape[1]
            dV = dV / g
        return dQ, dK, dV
    return backward


MUTATIONS = [
    ("_row_forward", _row_forward_no_scale),
    ("visible_keys", _visible_keys_no_inblock_mask),
    ("selected_set", _selected_set_drops_current),
    ("selected_set", _selected_set_multiset),
    ("backward", _backward_mutated("dk_unscaled")),
    ("backward", _backward_mutated("dq_sign")),
    ("backward", _backward_mutated("dv_one_head")),
]


def test_unmutated_oracle_passes_the_selected_pins():
    assert not _some_pin_fails()


@pytest.mark.parametrize("name,replacement", MUTATIONS, ids=[f"{n}-{i}" for i, (n, _) in enumerate(MUTATIONS)])
def test_planted_mistake_is_caught(monkeypatch, name, replacement):
    monkeypatch.setattr(orc, name, replacement)
    assert _some_pin_fails(), f"no pin noticed a broken {name}"


def test_inversion_mistake_is_caught(monkeypatch):
    real = orc.invert_index

    def descending(idx, cu, **kw):                      # lists in the wrong order
        cnt, off, qlist, qslot, vmask = real(idx, cu, **kw)
        for a, b in zip(off[:-1], off[1:]):
            qlist[a:b] = qlist[a:b][::-1].copy()
            qslot[a:b] = qslot[a:b][::-1].copy()
        return cnt, off, qlist, qslot, vmask
    monkeypatch.setattr(orc, "invert_index", descending)
    with pytest.raises(AssertionError):
        pins.test_inversion_against_mask_and_invariants(pins.CASES[0])


@pytest.mark.parametrize("kind", ["gate_not_applied_to_dO", "dgate_from_gated_output", "acc_dropped"])
def test_gated_combination_mistake_is_caught(monkeypatch, kind):
    real_fwd, real_bwd = orc.gated_forward, orc.gated_backward

    def fwd(O, gate, O_acc=None):
        return real_fwd(O, gate, None if kind == "acc_dropped" else O_acc)

    def bwd(Q, K, V, dO_out, gate, idx, cu, **kw):
        dQ, dK, dV, dgate = real_bwd(Q, K, V, dO_out, gate, idx, cu, **kw)
        if kind == "gate_not_applied_to_dO":
            dQ, dK, dV = orc.backward(Q, K, V, dO_out, idx, cu, **kw)
        if kind == "dgate_from_gated_output":
            dgate = dgate * gate
        return dQ, dK, dV, dgate
    pins.test_gated_combination_equals_autograd_of_dense_formulation()
    monkeypatch.setattr(orc, "gated_forward", fwd)
    monkeypatch.setattr(orc, "gated_backward", bwd)
    with pytest.raises(AssertionError):
        pins.test_gated_combination_equals_autograd_of_dense_formulation()


def test_window_off_by_one_is_caught(monkeypatch):
    real = orc.visible_keys

    def wider(cu, t, idx_row, block, causal, window=0):            # keeps u = t - window as well
        return real(cu, t, idx_row, block, causal, window + 1 if window else 0)
    pins.test_window_rows_give_banded_attention(100)
    monkeypatch.setattr(orc, "visible_keys", wider)
    with pytest.raises(AssertionError):
        pins.test_window_rows_give_banded_attention(100)
