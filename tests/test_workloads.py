"""The seeded generators: structure of the drawn index tables and bf16 plumbing."""
import numpy as np
import pytest

import workloads as wl


@pytest.mark.parametrize("name", wl.SMALL_NAMES + ["tiny"])
def test_rows_are_causal_distinct_and_forced(name):
    w = wl.realise(wl.small(name) if name != "tiny" else wl.named("tiny"), tensors=False)
    idx, cu = w.idx, w.cu_seqlens
    assert idx.shape == (w.total_tokens, w.hkv, w.topk) and idx.dtype == np.int32
    tok = np.arange(w.total_tokens)
    seq = np.searchsorted(cu, tok, side="right") - 1
    cur = (tok - cu[seq]) // w.block
    for t in range(0, w.total_tokens, 7):
        for j in range(w.hkv):
            row = idx[t, j]
            valid = row[row >= 0]
            assert len(set(valid.tolist())) == len(valid)                  # drawn without replacement
            assert np.all(valid <= cur[t])                                 # only the current and earlier blocks
            assert cur[t] in valid                                         # current block always there
            if w.sink:
                assert 0 in valid
            if w.recent == 2 and cur[t] >= 1:
                assert cur[t] - 1 in valid
            if w.local_picks == 0:
                assert len(valid) == min(w.topk, cur[t] + 1)               # padded only when blocks run out
            assert np.all(row[len(valid):] == -1)


def test_same_seed_same_data_and_bf16_round_trip():
    a = wl.realise(wl.small("g4"))
    b = wl.realise(wl.small("g4"))
    assert np.array_equal(a.idx, b.idx) and np.array_equal(a.q, b.q) and np.array_equal(a.do, b.do)
    x = np.array([1.0, 1.00390625, 1.01171875, -3.0e-40, 65504.0, 0.1], dtype=np.float32)
    bits = wl.f32_to_bf16_bits(x)
    back = wl.bf16_bits_to_f32(bits)
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == 1.015625      # ties to even, then round up
    assert np.all(np.abs(back[3:] - x[3:]) <= np.abs(x[3:]) * 2.0 ** -8 + 1e-38)
    assert np.array_equal(wl.f32_to_bf16_bits(back), bits)


def test_locality_skew_prefers_recent_blocks():
    w = wl.realise(wl.Workload("q", [4096], hq=7, hkv=1, topk=16, sink=True, local_picks=7, seed=5), tensors=False)
    t = 4000
    row = w.idx[t, 0]
    cur = t // 64
    recent = [x for x in row if cur - 8 <= x < cur]
    assert len(recent) == 7
