"""The paper's cost model (App. "FSA and NSA Theoretical Memory Access and FLOPs Analysis") and the effective
FLOP count the benchmark reports.  Plain arithmetic on shapes; no tensors."""
from __future__ import annotations


def fsa_selected_flops(N: int, h: int, d: int, B_K: int, T: int) -> float:
    """FLOPs of the KV-outer selected-attention kernel: 4 d h N B_K T (also the effective forward FLOPs)."""
    return 4.0 * d * h * N * B_K * T


def fsa_total_bytes(N: int, h: int, h_K: int, d: int, T: int) -> float:
    """Selected kernel 4dhN(1+T) + statistics pre-pass 2 d h_K N (1+T) + reduction 2dhN(1+T)."""
    return d * N * (6.0 * h + 2.0 * h_K) * (1 + T)


def fsa_total_flops(N: int, h: int, h_K: int, d: int, B_K: int, T: int) -> float:
    return d * N * B_K * T * (4.0 * h + 2.0 * h_K)


def nsa_bytes(N: int, h: int, h_K: int, d: int, B_K: int, T: int) -> float:
    """Query-outer NSA kernel: 2 d h_K N (B_K T + g + 8) bytes (heads padded to 8)."""
    g = h // h_K
    return 2.0 * d * h_K * N * (B_K * T + g + 8)


def nsa_flops(N: int, h_K: int, d: int, B_K: int, T: int) -> float:
    return 32.0 * d * h_K * N * B_K * T


def effective_flops(total_tokens: int, hq: int, topk: int, d: int = 128, block: int = 64):
    """(forward, backward) nominal FLOPs: 4 N h T B_K d forward, 2.5x that backward (5 GEMMs against 2);
    padded slots and the masked part of the diagonal block are counted."""
    f = fsa_selected_flops(total_tokens, hq, d, block, topk)
    return f, 2.5 * f


def compulsory_bytes(total_tokens: int, hq: int, hkv: int, topk: int, d: int = 128):
    """(forward, backward) bytes the method itself must move through HBM, each tensor once: forward reads Q, K, V and
    idx and writes O and LSE; backward reads Q, K, V, O, dO, LSE, delta and idx and writes dQ, dK, dV (bf16 tensors,
    fp32 row statistics, int32 idx).  Partial buffers and gathers re-reading Q / dO are not in it: they are what the
    measured traffic is compared against."""
    T = total_tokens
    stats, idx = 4.0 * T * hq, 4.0 * T * hkv * topk
    fwd = 2.0 * T * d * (2 * hq + 2 * hkv) + stats + idx
    bwd = 2.0 * T * d * (4 * hq + 4 * hkv) + 2 * stats + idx
    return fwd, bwd
