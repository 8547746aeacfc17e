"""Helpers of the GPU parity tests: upload a workload, run the library through its C ABI, compare."""
import numpy as np
import torch

import paper_2508_18224_amd as nsa
import workloads as wl

# spec tolerances, read as |gpu - ref| <= atol + rtol * |ref| per element, plus a Frobenius-norm bound
TOL_O = (2e-2, 1e-2)
TOL_GRAD = (4e-2, 2e-2)
TOL_LSE = 1e-3


def dev_bf16(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


class Case:
    """A realised workload on the device plus the library object that owns its workspaces."""

    def __init__(self, w: wl.Workload, bwd: bool = True, scale: float = 0.0, window: int = 0, dense: bool = True):
        self.w = w
        self.q, self.k, self.v, self.do = (dev_bf16(x) for x in (w.q, w.k, w.v, w.do))
        self.idx = torch.from_numpy(w.idx).cuda()
        self.cu = torch.from_numpy(w.cu_seqlens).cuda()
        self.attn = nsa.SelAttention(w.total_tokens, w.hq, w.hkv, w.topk, nseq=len(w.seqlens), causal=w.causal,
                                     scale=scale, bwd=bwd, block=w.block, window=window, dense=dense)

    def host_f64(self):
        w = self.w
        return tuple(wl.bf16_bits_to_f64(x) for x in (w.q, w.k, w.v, w.do))

    def forward(self, rebuild=True):
        o, lse = self.attn.forward(self.q, self.k, self.v, self.idx, self.cu, rebuild_index=rebuild)
        torch.cuda.synchronize()
        return o, lse

    def backward(self, o, lse):
        out = self.attn.backward(self.q, self.k, self.v, o, lse, self.do, self.cu)
        torch.cuda.synchronize()
        return out


def assert_close(name, got: np.ndarray, ref: np.ndarray, tol):
    atol, rtol = tol
    err = np.abs(got - ref)
    bound = atol + rtol * np.abs(ref)
    worst = float((err - bound).max()) if err.size else 0.0
    # the relative norm only means something when the reference is not itself (numerically) zero, e.g. the dQ of
    # a row with a single visible key is exactly 0
    ref_norm = float(np.linalg.norm(ref))
    fro = float(np.linalg.norm(err) / ref_norm) if err.size and ref_norm > atol * np.sqrt(err.size) * 1e-3 else 0.0
    assert worst <= 0, f"{name}: max-abs err {err.max():.4g} exceeds atol {atol} + rtol {rtol}*|ref| by {worst:.4g}"
    assert fro <= rtol, f"{name}: relative Frobenius error {fro:.4g} > {rtol}"
    return float(err.max()) if err.size else 0.0, fro


def assert_dgate_close(name, got: np.ndarray, dO: np.ndarray, O_ref: np.ndarray):
    """dgate[t, h] = <dO, O> is a 128-term dot product whose O factor the library holds in bf16: each product is off by
    at most half a bf16 ulp, 2^-9 relative, so the sum may be off by 2^-9 * sum_i |dO_i O_i| even where the sum itself
    cancels to ~0.  Bound: the gradient tolerance's absolute part plus twice that."""
    ref = (dO * O_ref).sum(axis=2)
    err = np.abs(got - ref)
    bound = TOL_GRAD[0] + 2.0 ** -8 * np.abs(dO * O_ref).sum(axis=2)
    worst = float((err - bound).max()) if err.size else 0.0
    assert worst <= 0, f"{name}: error exceeds 4e-2 + 2^-8 sum|dO O| by {worst:.4g}"


def assert_lse_close(got: np.ndarray, ref: np.ndarray):
    assert np.array_equal(np.isneginf(got), np.isneginf(ref)), "LSE: -inf pattern differs"
    fin = np.isfinite(ref)
    err = np.abs(got[fin] - ref[fin])
    assert err.size == 0 or err.max() <= TOL_LSE, f"LSE: max-abs err {err.max():.4g} > {TOL_LSE}"


class BitsF64:
    """bf16 bit patterns presented as a read-only float64 array that widens (exactly) only what is indexed,
    so that the oracle can sample a few rows of a multi-GB tensor."""

    def __init__(self, bits: np.ndarray):
        self.bits = bits
        self.shape = bits.shape
        self.dtype = np.dtype(np.float64)

    def __getitem__(self, ix):
        return wl.bf16_bits_to_f64(np.asarray(self.bits[ix]))
