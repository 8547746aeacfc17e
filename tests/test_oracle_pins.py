"""Pins for the CPU oracle: every check compares it with something that is not the oracle itself."""
import math

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import nsa_sel_oracle as orc

B = 64


def _rand_problem(seed, seqlens, hq, hkv, k, d=16, adversarial=False, **kw):
    rng = np.random.default_rng(seed)
    T = sum(seqlens)
    cu = np.concatenate([[0], np.cumsum(seqlens)]).astype(np.int32)
    if adversarial:
        idx = wl.draw_adversarial_indices(rng, seqlens, hkv, k)
    else:
        idx = wl.draw_block_indices(rng, seqlens, hkv, k, sink=kw.get("sink", False), recent=kw.get("recent", 1),
                                    local_picks=kw.get("local_picks", 0), local_window=8)
    Q = rng.standard_normal((T, hq, d))
    K = rng.standard_normal((T, hkv, d))
    V = rng.standard_normal((T, hkv, d))
    dO = rng.standard_normal((T, hq, d))
    return Q, K, V, dO, idx, cu


def _dense_mask(idx, cu, causal):
    """M[j, t, u] built by broadcasting straight from the definition (no per-token loops)."""
    T, hkv, k = idx.shape
    tok = np.arange(T)
    seq = np.searchsorted(cu, tok, side="right") - 1
    start = cu[seq]
    length = cu[seq + 1] - cu[seq]
    blk = (tok - start) // B                      # local block of every token (as key and as query)
    nblk = -(-length // B)
    M = np.zeros((hkv, T, T), dtype=bool)
    for j in range(hkv):
        ids = idx[:, j, :]                        # [T, k]
        ok = (ids >= 0) & (ids < nblk[:, None])
        if causal:
            ok &= ids <= blk[:, None]
        hit = (ids[:, :, None] == blk[None, None, :]) & ok[:, :, None]      # [T, k, U]
        m = hit.any(axis=1) & (seq[:, None] == seq[None, :])
        if causal:
            m &= tok[None, :] <= tok[:, None]
        M[j] = m
    return M


def _dense_forward_np(Q, K, V, M, scale):
    T, hq, d = Q.shape
    hkv = K.shape[1]
    g = hq // hkv
    O = np.zeros_like(Q)
    LSE = np.full((T, hq), -np.inf)
    for h in range(hq):
        j = h // g
        S = scale * Q[:, h] @ K[:, j].T
        S = np.where(M[j], S, -np.inf)
        mx = S.max(axis=1, keepdims=True)
        ok = np.isfinite(mx[:, 0])
        E = np.exp(S[ok] - mx[ok])
        L = E.sum(axis=1, keepdims=True)
        O[ok, h] = (E / L) @ V[:, j]
        LSE[ok, h] = (mx[ok] + np.log(L))[:, 0]
    return O, LSE


def _dense_torch(Q, K, V, M, scale):
    """Dense masked attention written with torch ops so that autograd supplies the gradients."""
    T, hq, d = Q.shape
    g = hq // K.shape[1]
    Kr = K.repeat_interleave(g, dim=1)
    Vr = V.repeat_interleave(g, dim=1)
    Mr = torch.from_numpy(M).repeat_interleave(g, dim=0)                    # [hq, T, U]
    S = scale * torch.einsum("thd,uhd->htu", Q, Kr)
    S = S.masked_fill(~Mr, float("-inf"))
    P = torch.softmax(S, dim=-1)
    P = torch.nan_to_num(P, nan=0.0)
    return torch.einsum("htu,uhd->thd", P, Vr)


CASES = [
    dict(seed=1, seqlens=[300], hq=4, hkv=1, k=4, causal=True),
    dict(seed=2, seqlens=[130, 1, 77, 200], hq=6, hkv=2, k=3, causal=True),
    dict(seed=3, seqlens=[257], hq=7, hkv=1, k=5, causal=True, sink=True, recent=2),
    dict(seed=4, seqlens=[190, 66], hq=2, hkv=2, k=6, causal=False, adversarial=True),
    dict(seed=5, seqlens=[200], hq=8, hkv=1, k=6, causal=True, adversarial=True),
]


@pytest.mark.parametrize("case", CASES)
def test_forward_equals_dense_masked_attention(case):
    case = dict(case)
    causal = case.pop("causal")
    Q, K, V, dO, idx, cu = _rand_problem(**case)
    scale = 0.37
    O, LSE = orc.forward(Q, K, V, idx, cu, causal=causal, scale=scale)
    M = _dense_mask(idx, cu, causal)
    O2, LSE2 = _dense_forward_np(Q, K, V, M, scale)
    assert np.array_equal(np.isfinite(LSE), np.isfinite(LSE2))
    np.testing.assert_allclose(O, O2, rtol=0, atol=1e-12)
    fin = np.isfinite(LSE2)
    np.testing.assert_allclose(LSE[fin], LSE2[fin], rtol=0, atol=1e-12)


@pytest.mark.parametrize("case", CASES)
def test_backward_equals_autograd_of_dense_masked_attention(case):
    case = dict(case)
    causal = case.pop("causal")
    Q, K, V, dO, idx, cu = _rand_problem(**case)
    scale = 0.21
    dQ, dK, dV = orc.backward(Q, K, V, dO, idx, cu, causal=causal, scale=scale)
    M = _dense_mask(idx, cu, causal)
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (Q, K, V))
    out = _dense_torch(tq, tk, tv, M, scale)
    out.backward(torch.from_numpy(dO))
    np.testing.assert_allclose(dQ, tq.grad.numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(dK, tk.grad.numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(dV, tv.grad.numpy(), rtol=0, atol=1e-11)


def test_gated_combination_equals_autograd_of_dense_formulation():
    """Eq. (2): out = acc + gate * attention.  Forward and all four gradients against torch autograd of the dense
    masked formulation; a zero gate must switch the branch (and its gradients) off."""
    Q, K, V, dO, idx, cu = _rand_problem(31, [130, 90], hq=4, hkv=2, k=3)
    rng = np.random.default_rng(32)
    gate = rng.random(Q.shape[:2])
    gate[5] = 0.0
    acc = rng.standard_normal(Q.shape)
    scale = 0.3
    O, _ = orc.forward(Q, K, V, idx, cu, scale=scale)
    out = orc.gated_forward(O, gate, acc)
    dQ, dK, dV, dgate = orc.gated_backward(Q, K, V, dO, gate, idx, cu, scale=scale)
    M = _dense_mask(idx, cu, True)
    tq, tk, tv, tg = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (Q, K, V, gate))
    tout = torch.from_numpy(acc) + tg[:, :, None] * _dense_torch(tq, tk, tv, M, scale)
    np.testing.assert_allclose(out, tout.detach().numpy(), rtol=0, atol=1e-12)
    tout.backward(torch.from_numpy(dO))
    np.testing.assert_allclose(dQ, tq.grad.numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(dK, tk.grad.numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(dV, tv.grad.numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(dgate, tg.grad.numpy(), rtol=0, atol=1e-11)
    assert not dQ[5].any()
    np.testing.assert_array_equal(orc.gated_forward(O, gate)[5], 0.0)


def _band_mask(cu, hkv, window):
    T = int(cu[-1])
    tok = np.arange(T)
    seq = np.searchsorted(cu, tok, side="right") - 1
    m = (seq[:, None] == seq[None, :]) & (tok[None, :] <= tok[:, None]) & (tok[None, :] > tok[:, None] - window)
    return np.broadcast_to(m, (hkv, T, T)).copy()


@pytest.mark.parametrize("window", [1, 64, 100, 129, 1000])
def test_window_rows_give_banded_attention(window):
    """The sliding-window term of Eq. (2): with idx listing the blocks the window touches and window = w, forward
    and backward equal dense attention under the band mask t - w < u <= t (torch softmax + autograd)."""
    seqlens = [300, 70, 1, 200]
    rng = np.random.default_rng(40 + window)
    T, hq, hkv, d = sum(seqlens), 4, 2, 16
    cu = np.concatenate([[0], np.cumsum(seqlens)]).astype(np.int32)
    idx = wl.window_block_indices(seqlens, hkv, window)
    Q, K, V, dO = (rng.standard_normal((T, h, d)) for h in (hq, hkv, hkv, hq))
    scale = 0.25
    O, LSE = orc.forward(Q, K, V, idx, cu, scale=scale, window=window)
    dQ, dK, dV = orc.backward(Q, K, V, dO, idx, cu, scale=scale, window=window)
    M = _band_mask(cu, hkv, window)
    O2, LSE2 = _dense_forward_np(Q, K, V, M, scale)
    np.testing.assert_allclose(O, O2, rtol=0, atol=1e-12)
    np.testing.assert_allclose(LSE, LSE2, rtol=0, atol=1e-12)
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (Q, K, V))
    _dense_torch(tq, tk, tv, M, scale).backward(torch.from_numpy(dO))
    np.testing.assert_allclose(dQ, tq.grad.numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(dK, tk.grad.numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(dV, tv.grad.numpy(), rtol=0, atol=1e-11)


def test_window_drops_blocks_wholly_outside_and_inversion_follows():
    """A listed (token, block) pair survives the inversion exactly when the block holds a key inside the window."""
    seqlens = [400, 130]
    window = 100
    cu = np.concatenate([[0], np.cumsum(seqlens)]).astype(np.int32)
    rng = np.random.default_rng(50)
    idx = wl.draw_block_indices(rng, seqlens, 2, 5, sink=True, recent=2, local_picks=2, local_window=4)
    cnt, off, qlist, qslot, vmask = orc.invert_index(idx, cu, window=window)
    M = _dense_mask(idx, cu, True) & _band_mask(cu, 2, window)
    nblk = [-(-L // B) for L in seqlens]
    base = [0, nblk[0]]
    for j in range(2):
        for s in range(2):
            for x in range(nblk[s]):
                lst = qlist[off[j * sum(nblk) + base[s] + x]: off[j * sum(nblk) + base[s] + x + 1]]
                keys = slice(int(cu[s]) + x * B, min(int(cu[s]) + (x + 1) * B, int(cu[s + 1])))
                expect = np.nonzero(M[j][:, keys].any(axis=1))[0]
                assert np.array_equal(lst, expect), (j, s, x)
    assert cnt.sum() < orc.invert_index(idx, cu)[0].sum()       # the window did drop pairs


@pytest.mark.parametrize("causal", [True, False])
def test_all_blocks_selected_is_full_attention(causal):
    """Top-k covering every block reduces the sel branch to Eq. (1); torch's SDPA is the library routine."""
    rng = np.random.default_rng(7)
    T, hq, hkv, d = 250, 6, 3, 32
    nb = -(-T // B)
    Q, K, V = (rng.standard_normal((T, h, d)) for h in (hq, hkv, hkv))
    idx = np.tile(rng.permutation(nb).astype(np.int32), (T, hkv, 1))
    cu = np.array([0, T], dtype=np.int32)
    O, LSE = orc.forward(Q, K, V, idx, cu, causal=causal)
    g = hq // hkv
    tq = torch.from_numpy(Q).permute(1, 0, 2)
    tk = torch.from_numpy(K).repeat_interleave(g, dim=1).permute(1, 0, 2)
    tv = torch.from_numpy(V).repeat_interleave(g, dim=1).permute(1, 0, 2)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=causal).permute(1, 0, 2).numpy()
    np.testing.assert_allclose(O, ref, rtol=0, atol=1e-12)
    S = torch.einsum("htd,hud->htu", tq, tk) / math.sqrt(d)
    if causal:
        S = S.masked_fill(torch.ones(T, T, dtype=torch.bool).triu(1), float("-inf"))
    np.testing.assert_allclose(LSE, torch.logsumexp(S, dim=-1).T.numpy(), rtol=0, atol=1e-12)


def test_backward_matches_central_finite_differences():
    Q, K, V, dO, idx, cu = _rand_problem(21, [150, 70], hq=4, hkv=2, k=3, d=8)
    W = dO
    scale = 0.5

    def loss(q, k, v):
        O, _ = orc.forward(q, k, v, idx, cu, scale=scale)
        return float((O * W).sum())

    dQ, dK, dV = orc.backward(Q, K, V, W, idx, cu, scale=scale)
    rng = np.random.default_rng(0)
    eps = 1e-6
    for name, X, G in (("q", Q, dQ), ("k", K, dK), ("v", V, dV)):
        for _ in range(12):
            pos = tuple(int(rng.integers(0, n)) for n in X.shape)
            Xp, Xm = X.copy(), X.copy()
            Xp[pos] += eps
            Xm[pos] -= eps
            args_p = {"q": (Xp, K, V), "k": (Q, Xp, V), "v": (Q, K, Xp)}[name]
            args_m = {"q": (Xm, K, V), "k": (Q, Xm, V), "v": (Q, K, Xm)}[name]
            fd = (loss(*args_p) - loss(*args_m)) / (2 * eps)
            assert abs(fd - G[pos]) <= 1e-6 * max(1.0, abs(fd)), (name, pos, fd, G[pos])


def test_closed_forms():
    Q, K, V, dO, idx, cu = _rand_problem(31, [333, 129], hq=4, hkv=2, k=5, d=16, sink=True)
    T = Q.shape[0]
    # (a) equal value rows: the output is that row whatever is selected
    v = np.linspace(-1, 1, 16)
    O, _ = orc.forward(Q, K, np.broadcast_to(v, V.shape).copy(), idx, cu)
    np.testing.assert_allclose(O, np.broadcast_to(v, O.shape), atol=1e-13)
    # (b) zero queries: LSE = ln(number of visible keys), a count fixed by the drop and mask rules
    _, LSE = orc.forward(np.zeros_like(Q), K, V, idx, cu)
    for t in range(T):
        s = int(np.searchsorted(cu, t, side="right") - 1)
        p = t - cu[s]
        cur = p // B
        for j in range(2):
            ids = {int(x) for x in idx[t, j] if 0 <= x <= cur}
            n = sum(B for x in ids if x < cur) + (p % B + 1 if cur in ids else 0)
            assert abs(LSE[t, 2 * j] - math.log(n)) < 1e-13
    # (c) softmax rows sum to one: column sums of dV equal the summed dO of each group
    dQ, dK, dV = orc.backward(Q, K, V, dO, idx, cu)
    np.testing.assert_allclose(dV.sum(axis=0), dO.reshape(T, 2, 2, 16).sum(axis=(0, 2)), atol=1e-10)
    # (d) equal key rows: scores are constant along a row, so dQ vanishes
    dQ2, _, _ = orc.backward(Q, np.broadcast_to(v, K.shape).copy(), V, dO, idx, cu)
    np.testing.assert_allclose(dQ2, 0, atol=1e-12)
    # (e) column order of idx does not matter; repeated ids count once
    perm = np.random.default_rng(5).permutation(idx.shape[2])
    O1, L1 = orc.forward(Q, K, V, idx, cu)
    O2, L2 = orc.forward(Q, K, V, idx[:, :, perm], cu)
    np.testing.assert_allclose(O1, O2, atol=1e-13)
    O3, L3 = orc.forward(Q, K, V, np.concatenate([idx, idx], axis=2), cu)
    np.testing.assert_allclose(O1, O3, atol=1e-13)
    np.testing.assert_allclose(L1, L3, atol=1e-13)


def test_single_current_block_is_block_diagonal_causal_attention():
    rng = np.random.default_rng(9)
    T, d = 200, 8
    Q, K, V = (rng.standard_normal((T, 1, d)) for _ in range(3))
    idx = (np.arange(T) // B).astype(np.int32).reshape(T, 1, 1)
    cu = np.array([0, T], dtype=np.int32)
    O, _ = orc.forward(Q, K, V, idx, cu)
    for b0 in range(0, T, B):
        sl = slice(b0, min(b0 + B, T))
        q, k, v = (torch.from_numpy(x[sl, 0]) for x in (Q, K, V))
        ref = torch.nn.functional.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True)[0]
        np.testing.assert_allclose(O[sl, 0], ref.numpy(), atol=1e-12)


def test_empty_rows_and_no_gradient_from_them():
    rng = np.random.default_rng(3)
    T, d = 100, 8
    Q, K, V, dO = (rng.standard_normal((T, 2, d)) for _ in range(4))
    idx = np.full((T, 2, 3), -1, dtype=np.int32)
    idx[:, 1, 0] = 5                       # future / out-of-range block for every token (T = 100 has 2 blocks)
    idx[70:, 0, 1] = 0
    cu = np.array([0, T], dtype=np.int32)
    O, LSE = orc.forward(Q, K, V, idx, cu)
    assert np.all(O[:70] == 0) and np.all(np.isneginf(LSE[:70])) and np.all(np.isneginf(LSE[:, 1]))
    dQ, dK, dV = orc.backward(Q, K, V, dO, idx, cu)
    assert np.all(dQ[:70] == 0) and np.all(dK[:, 1] == 0) and np.all(dV[64:] == 0)


@pytest.mark.parametrize("case", CASES)
def test_inversion_against_mask_and_invariants(case):
    case = dict(case)
    causal = case.pop("causal")
    Q, K, V, dO, idx, cu = _rand_problem(**case)
    T, hkv, k = idx.shape
    cnt, off, qlist, qslot, vmask = orc.invert_index(idx, cu, causal=causal)
    tok = np.arange(T)
    seq = np.searchsorted(cu, tok, side="right") - 1
    length = cu[seq + 1] - cu[seq]
    blk = (tok - cu[seq]) // B
    nblk_seq = -(-np.diff(cu) // B)
    base = np.concatenate([[0], np.cumsum(nblk_seq)])
    b_tot = int(base[-1])
    assert cnt.shape == (hkv, b_tot) and off[-1] == cnt.sum() == len(qlist) == len(qslot)
    for j in range(hkv):
        ids = idx[:, j, :].astype(np.int64)
        ok = (ids >= 0) & (ids < (-(-length // B))[:, None])
        if causal:
            ok &= ids <= blk[:, None]
        gid = np.where(ok, ids + base[seq][:, None], -1)
        for gb in range(b_tot):
            want = np.nonzero((gid == gb).any(axis=1))[0]
            lo, hi = off[j * b_tot + gb], off[j * b_tot + gb + 1]
            assert hi - lo == cnt[j, gb]
            assert np.array_equal(qlist[lo:hi], want)                       # ascending, each token once
            for t, m in zip(qlist[lo:hi], qslot[lo:hi]):
                assert gid[t, m] == gb and not (gid[t, :m] == gb).any()     # first occurrence
                assert (vmask[t, j] >> m) & 1
    assert sum(bin(int(x)).count("1") for x in vmask.reshape(-1)) == len(qlist)


def test_sink_list_holds_every_token():
    w = wl.realise(wl.Workload("s", [640], hq=2, hkv=2, topk=6, sink=True, seed=3), tensors=False)
    cnt, off, qlist, qslot, _ = orc.invert_index(w.idx, w.cu_seqlens)
    assert np.all(cnt[:, 0] == 640)
    assert np.array_equal(qlist[off[0]:off[1]], np.arange(640))


def test_backward_kv_blocks_matches_full_backward():
    Q, K, V, dO, idx, cu = _rand_problem(41, [200, 131], hq=4, hkv=2, k=4, d=8, sink=True)
    dQ, dK, dV = orc.backward(Q, K, V, dO, idx, cu)
    blocks = [(0, 0, 0), (1, 0, 3), (0, 1, 2), (1, 1, 0)]
    got = orc.backward_kv_blocks(Q, K, V, dO, idx, cu, blocks)
    for (j, s, x), (dKb, dVb) in zip(blocks, got):
        lo = cu[s] + x * B
        hi = min(lo + B, cu[s + 1])
        np.testing.assert_allclose(dKb, dK[lo:hi, j], atol=1e-12)
        np.testing.assert_allclose(dVb, dV[lo:hi, j], atol=1e-12)
