"""ctypes marshalling for include/nsa_sel.h.  No arithmetic happens here."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libnsa_sel.so")
_lib = None

SYMBOLS = ["nsa_sel_workspace_bytes", "nsa_sel_workspace_bytes_min", "nsa_sel_build_index", "nsa_sel_index_view", "nsa_sel_fwd", "nsa_sel_bwd", "nsa_sel_fwd_static", "nsa_sel_fwd_query_outer", "nsa_sel_fwd_gated", "nsa_sel_bwd_gated", "nsa_sel_select_blocks",
           "nsa_sel_profile_enable", "nsa_sel_profile_select", "nsa_sel_profile_collect", "nsa_sel_calibration_copy", "nsa_sel_mfma_probe", "nsa_sel_strerror"]


class NsaSelError(RuntimeError):
    pass


class Shape(C.Structure):
    _fields_ = [("total_tokens", C.c_int32), ("nseq", C.c_int32), ("hq", C.c_int32), ("hkv", C.c_int32),
                ("d", C.c_int32), ("block", C.c_int32), ("topk", C.c_int32), ("causal", C.c_int32),
                ("scale", C.c_float), ("max_seqlen", C.c_int32), ("window", C.c_int32), ("unit", C.c_int32),
                ("dense", C.c_int32)]


def lib():
    """Load the built library (raises if it has not been built; see paper_2508_18224_amd/build.py)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise NsaSelError(f"{_LIB_PATH} is missing: run `python -m paper_2508_18224_amd.build` first")
        L = C.CDLL(_LIB_PATH)
        vp, sz, i32p = C.c_void_p, C.c_size_t, C.c_void_p
        L.nsa_sel_workspace_bytes.argtypes = [C.POINTER(Shape), C.POINTER(sz), C.POINTER(sz), C.POINTER(sz)]
        L.nsa_sel_workspace_bytes_min.argtypes = [C.POINTER(Shape), C.POINTER(sz), C.POINTER(sz)]
        L.nsa_sel_build_index.argtypes = [C.POINTER(Shape), i32p, i32p, vp, sz, vp]
        L.nsa_sel_index_view.argtypes = [C.POINTER(Shape), vp] + [C.POINTER(vp)] * 4 + [C.POINTER(C.c_int32)]
        L.nsa_sel_fwd.argtypes = [C.POINTER(Shape), vp, vp, vp, i32p, i32p, C.c_int, vp, sz, vp, vp, vp, sz, vp]
        L.nsa_sel_bwd.argtypes = [C.POINTER(Shape), vp, vp, vp, vp, vp, vp, i32p, vp, sz, vp, vp, vp, vp, sz, vp]
        L.nsa_sel_fwd_static.argtypes = [C.POINTER(Shape), vp, vp, vp, i32p, i32p, C.c_int, vp, sz, vp, vp, vp]
        L.nsa_sel_fwd_query_outer.argtypes = [C.POINTER(Shape), vp, vp, vp, i32p, i32p, vp, vp, vp]
        L.nsa_sel_fwd_gated.argtypes = [C.POINTER(Shape), vp, vp, vp, i32p, i32p, C.c_int, vp, sz, vp, vp, vp, vp, vp, vp, sz, vp]
        L.nsa_sel_bwd_gated.argtypes = [C.POINTER(Shape), vp, vp, vp, vp, vp, vp, vp, i32p, vp, sz, vp, vp, vp, vp, vp, sz, vp]
        L.nsa_sel_select_blocks.argtypes = [C.POINTER(Shape), vp, C.c_int64, i32p, C.c_int32, C.c_int32, i32p, vp]
        L.nsa_sel_profile_enable.argtypes = [C.c_int]
        L.nsa_sel_profile_select.argtypes = [C.c_uint]
        L.nsa_sel_profile_collect.argtypes = [C.c_int, C.POINTER(C.c_char_p), C.POINTER(C.c_float),
                                              C.POINTER(C.c_int)]
        L.nsa_sel_calibration_copy.argtypes = [vp, vp, sz, vp]
        L.nsa_sel_mfma_probe.argtypes = [C.c_int, vp, C.POINTER(C.c_double), vp]
        L.nsa_sel_strerror.argtypes = [C.c_int]
        L.nsa_sel_strerror.restype = C.c_char_p
        for name in SYMBOLS[:-1]:
            getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def _check(rc: int, what: str):
    if rc != 0:
        raise NsaSelError(f"{what}: {lib().nsa_sel_strerror(rc).decode()} ({rc})")


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise NsaSelError("tensors must be contiguous device tensors")
    return C.c_void_p(t.data_ptr())


def _stream(device=None):
    """The current stream of `device` (of the current device when None), as the void* the C ABI takes."""
    return C.c_void_p(torch.cuda.current_stream(device).cuda_stream)


def _nbytes(t: torch.Tensor) -> int:
    return t.numel() * t.element_size()


def _device(device) -> torch.device:
    """torch.device with an explicit index ("cuda" means the current device)."""
    d = torch.device(device)
    if d.type == "cuda" and d.index is None:
        d = torch.device("cuda", torch.cuda.current_device())
    return d


def expect_tensor(name: str, t, dtype, shape, device, optional: bool = False):
    """Host-side check of one tensor argument before its address is handed to the library: the kernels trust
    dtype, extent and device, so a wrong one would be read or written out of bounds."""
    if t is None:
        if optional:
            return
        raise NsaSelError(f"{name} is required")
    if not isinstance(t, torch.Tensor):
        raise NsaSelError(f"{name} must be a torch.Tensor")
    if t.dtype != dtype:
        raise NsaSelError(f"{name} must be {dtype}, got {t.dtype}")
    if tuple(t.shape) != tuple(shape):
        raise NsaSelError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")
    if t.device != _device(device):
        raise NsaSelError(f"{name} must live on {_device(device)}, got {t.device}")
    if not t.is_contiguous():
        raise NsaSelError(f"{name} must be contiguous")


def expect_workspace(name: str, t, min_bytes: int, device):
    if not isinstance(t, torch.Tensor) or t.device != _device(device) or not t.is_contiguous():
        raise NsaSelError(f"{name} must be a contiguous tensor on {_device(device)}")
    if _nbytes(t) < min_bytes:
        raise NsaSelError(f"{name} holds {_nbytes(t)} bytes, {min_bytes} are needed")


def expect_attention_args(s: "Shape", device, *, q=None, k=None, v=None, idx=None, cu=None, o=None, lse=None,
                          do=None, grads=None, gate=None, o_acc=None, o_out=None, dgate=None, need_idx=False):
    """dtype / shape / device of every tensor of a forward or backward call against the shape `s` (only the
    tensors given are checked; cu is required when the shape packs several sequences)."""
    T, hq, hkv, d = s.total_tokens, s.hq, s.hkv, s.d
    bf, f32, i32 = torch.bfloat16, torch.float32, torch.int32
    for name, t, heads in (("q", q, hq), ("k", k, hkv), ("v", v, hkv), ("o", o, hq), ("do", do, hq),
                           ("o_acc", o_acc, hq), ("o_out", o_out, hq)):
        expect_tensor(name, t, bf, (T, heads, d), device, optional=True)
    expect_tensor("lse", lse, f32, (T, hq), device, optional=True)
    expect_tensor("gate", gate, f32, (T, hq), device, optional=True)
    expect_tensor("dgate", dgate, f32, (T, hq), device, optional=True)
    expect_tensor("idx", idx, i32, (T, hkv, s.topk), device, optional=not need_idx)
    expect_tensor("cu_seqlens", cu, i32, (s.nseq + 1,), device, optional=s.nseq == 1)
    if grads is not None:
        for name, t, heads in zip(("dq", "dk", "dv"), grads, (hq, hkv, hkv)):
            expect_tensor(name, t, bf, (T, heads, d), device)
    if o_out is not None and o is not None and o_out.data_ptr() == o.data_ptr() and T > 0:
        raise NsaSelError("o_out must not be the tensor o")
    if o_acc is not None and o is not None and o_acc.data_ptr() == o.data_ptr() and T > 0:
        raise NsaSelError("o_acc must not be the tensor o (the result would be o + gate * o)")


def workspace_bytes(shape: Shape):
    f, b, i = C.c_size_t(), C.c_size_t(), C.c_size_t()
    _check(lib().nsa_sel_workspace_bytes(C.byref(shape), C.byref(f), C.byref(b), C.byref(i)), "nsa_sel_workspace_bytes")
    return f.value, b.value, i.value


def workspace_bytes_min(shape: Shape):
    """Smallest (forward, backward) workspaces the library accepts: one KV head per pass."""
    f, b = C.c_size_t(), C.c_size_t()
    _check(lib().nsa_sel_workspace_bytes_min(C.byref(shape), C.byref(f), C.byref(b)), "nsa_sel_workspace_bytes_min")
    return f.value, b.value


def build_index(shape: Shape, idx: torch.Tensor, cu: Optional[torch.Tensor], index_ws: torch.Tensor):
    dev = index_ws.device
    expect_attention_args(shape, dev, idx=idx, cu=cu, need_idx=True)
    expect_workspace("index_ws", index_ws, workspace_bytes(shape)[2], dev)
    with torch.cuda.device(dev):
        _check(lib().nsa_sel_build_index(C.byref(shape), _ptr(idx), _ptr(cu), _ptr(index_ws), _nbytes(index_ws),
                                         _stream(dev)), "nsa_sel_build_index")


def index_view(shape: Shape, index_ws: torch.Tensor):
    """Byte offsets (from the workspace base) of cnt, off, qent, vmask, and the list stride b_cap."""
    outs = [C.c_void_p() for _ in range(4)]
    bcap = C.c_int32()
    _check(lib().nsa_sel_index_view(C.byref(shape), _ptr(index_ws), *[C.byref(o) for o in outs], C.byref(bcap)),
           "nsa_sel_index_view")
    base = index_ws.data_ptr()
    return [o.value - base for o in outs], bcap.value


def nsa_sel_fwd(shape, q, k, v, idx, cu, rebuild_index, index_ws, o, lse, ws):
    dev = index_ws.device
    expect_attention_args(shape, dev, q=q, k=k, v=v, idx=idx, cu=cu, o=o, lse=lse, need_idx=bool(rebuild_index))
    expect_workspace("index_ws", index_ws, workspace_bytes(shape)[2], dev)
    expect_workspace("ws", ws, workspace_bytes_min(shape)[0], dev)
    with torch.cuda.device(dev):
        _check(lib().nsa_sel_fwd(C.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ptr(idx), _ptr(cu), int(rebuild_index),
                                 _ptr(index_ws), _nbytes(index_ws), _ptr(o), _ptr(lse), _ptr(ws), _nbytes(ws),
                                 _stream(dev)), "nsa_sel_fwd")


def nsa_sel_fwd_static(shape, q, k, v, idx, cu, rebuild_index, index_ws, o, lse):
    """nsa_sel_fwd with the partial buffers in the library's own device array (no workspace argument)."""
    dev = index_ws.device
    expect_attention_args(shape, dev, q=q, k=k, v=v, idx=idx, cu=cu, o=o, lse=lse, need_idx=bool(rebuild_index))
    expect_workspace("index_ws", index_ws, workspace_bytes(shape)[2], dev)
    with torch.cuda.device(dev):
        _check(lib().nsa_sel_fwd_static(C.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ptr(idx), _ptr(cu),
                                        int(rebuild_index), _ptr(index_ws), _nbytes(index_ws), _ptr(o), _ptr(lse),
                                        _stream(dev)), "nsa_sel_fwd_static")


def nsa_sel_bwd(shape, q, k, v, o, lse, do, cu, index_ws, dq, dk, dv, ws):
    dev = index_ws.device
    expect_attention_args(shape, dev, q=q, k=k, v=v, cu=cu, o=o, lse=lse, do=do, grads=(dq, dk, dv))
    expect_workspace("index_ws", index_ws, workspace_bytes(shape)[2], dev)
    expect_workspace("ws", ws, workspace_bytes_min(shape)[1], dev)
    with torch.cuda.device(dev):
        _check(lib().nsa_sel_bwd(C.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(do), _ptr(cu),
                                 _ptr(index_ws), _nbytes(index_ws), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(ws), _nbytes(ws),
                                 _stream(dev)), "nsa_sel_bwd")


def select_blocks(scores: torch.Tensor, cu: Optional[torch.Tensor], topk: int, *, block: int = 64,
                  causal: bool = True, n_sink: int = 1, n_local: int = 2, out: Optional[torch.Tensor] = None):
    """idx int32 [tokens, hkv, topk] from fp32 scores [tokens, hkv, stride] (nsa_sel_select_blocks)."""
    if scores.dtype != torch.float32 or scores.dim() != 3:
        raise NsaSelError("scores must be float32 [tokens, hkv, stride]")
    T, hkv, stride = scores.shape
    nseq = 1 if cu is None else cu.numel() - 1
    shape = Shape(T, nseq, hkv, hkv, 128, block, topk, int(causal), 0.0, 0)
    dev = scores.device
    if out is None:
        out = torch.empty(T, hkv, topk, dtype=torch.int32, device=dev)
    expect_tensor("scores", scores, torch.float32, (T, hkv, stride), dev)
    expect_tensor("cu_seqlens", cu, torch.int32, (nseq + 1,), dev, optional=True)
    expect_tensor("out", out, torch.int32, (T, hkv, topk), dev)
    with torch.cuda.device(dev):
        _check(lib().nsa_sel_select_blocks(C.byref(shape), _ptr(scores), stride, _ptr(cu), n_sink, n_local, _ptr(out),
                                           _stream(dev)), "nsa_sel_select_blocks")
    return out


def window_blocks(total_tokens: int, hkv: int, window: int, cu: Optional[torch.Tensor] = None, *, block: int = 64,
                  device="cuda:0"):
    """idx int32 [tokens, hkv, R + 1], R = ceil((window - 1) / block): the blocks a causal window of `window` tokens
    can touch, most recent first (nsa_sel_select_blocks with no scores: forced local blocks only)."""
    topk = -(-(window - 1) // block) + 1
    nseq = 1 if cu is None else cu.numel() - 1
    shape = Shape(total_tokens, nseq, hkv, hkv, 128, block, topk, 1, 0.0, 0)
    dev = _device(device)
    out = torch.empty(total_tokens, hkv, topk, dtype=torch.int32, device=dev)
    expect_tensor("cu_seqlens", cu, torch.int32, (nseq + 1,), dev, optional=True)
    with torch.cuda.device(dev):
        _check(lib().nsa_sel_select_blocks(C.byref(shape), None, 0, _ptr(cu), 0, topk, _ptr(out), _stream(dev)),
               "nsa_sel_select_blocks")
    return out


def profile_enable(capacity: int):
    _check(lib().nsa_sel_profile_enable(int(capacity)), "nsa_sel_profile_enable")


def profile_select(names=None):
    """Record only the named kernel kinds (None: all).  Names are those profile_collect reports; call it before
    recording starts (it drops launches recorded so far)."""
    if names is None:
        mask = 0xFFFFFFFF
    else:
        order = list(profile_collect())
        mask = 0
        for nm in names:
            mask |= 1 << order.index(nm)
    _check(lib().nsa_sel_profile_select(mask), "nsa_sel_profile_select")


def profile_collect():
    """{kernel name: (total ms, launches)} of the launches recorded since the last collect."""
    n = 32
    names = (C.c_char_p * n)()
    ms = (C.c_float * n)()
    calls = (C.c_int * n)()
    got = lib().nsa_sel_profile_collect(n, names, ms, calls)
    if got < 0:
        _check(got, "nsa_sel_profile_collect")
    return {names[i].decode(): (float(ms[i]), int(calls[i])) for i in range(got)}


def calibration_copy(dst: torch.Tensor, src: torch.Tensor):
    nbytes = _nbytes(src)
    if _nbytes(dst) < nbytes or dst.device != src.device:
        raise NsaSelError("calibration_copy: dst must be on src's device and at least as large")
    with torch.cuda.device(src.device):
        _check(lib().nsa_sel_calibration_copy(_ptr(dst), _ptr(src), nbytes, _stream(src.device)),
               "nsa_sel_calibration_copy")


def mfma_probe(iters: int, sink: torch.Tensor) -> float:
    """Enqueue the MFMA probe kernel; returns the FLOPs it performs."""
    fl = C.c_double()
    expect_tensor("sink", sink, torch.float32, tuple(sink.shape), sink.device)
    with torch.cuda.device(sink.device):
        _check(lib().nsa_sel_mfma_probe(int(iters), _ptr(sink), C.byref(fl), _stream(sink.device)), "nsa_sel_mfma_probe")
    return fl.value


class SelAttention:
    """Owns the workspaces for one shape and calls the library (buffers are torch uint8 tensors)."""

    def __init__(self, total_tokens, hq, hkv, topk, *, nseq=1, causal=True, scale=0.0, device="cuda:0", bwd=True,
                 block=64, ws_cap_bytes=None, window=0, unit=0, dense=None):
        """ws_cap_bytes caps each of the forward / backward workspaces (never below the library's minimum);
        the library then works through the KV heads in as many passes as needed.  dense: None lets the library
        route the forward (shape.dense = 0), True / False force the dense route on / off."""
        self.shape = Shape(total_tokens, nseq, hq, hkv, 128, block, topk, int(causal), float(scale), 0, int(window),
                           int(unit), 0 if dense is None else (1 if dense else -1))
        fb, bb, ib = workspace_bytes(self.shape)
        if ws_cap_bytes is not None:
            fmin, bmin = workspace_bytes_min(self.shape)
            fb = min(fb, max(fmin, int(ws_cap_bytes)))
            bb = min(bb, max(bmin, int(ws_cap_bytes)))
        self.device = _device(device)
        self.index_ws = torch.empty(ib, dtype=torch.uint8, device=self.device)
        self.fwd_ws = torch.empty(fb, dtype=torch.uint8, device=self.device)
        self.bwd_ws = torch.empty(bb, dtype=torch.uint8, device=self.device) if bwd else None

    @classmethod
    def autotuned(cls, q, k, v, idx, do, cu=None, *, topk, candidates=(256, 512, 1024, 2048), reps=3, **kw):
        """The paper picks its query batch size by timing the candidates once per configuration (App. E); this does
        the same for the work-unit size: builds one object per candidate, times `reps` forward + backward steps on
        the given tensors with device events, and returns (best object, {unit: ms})."""
        T, hq = q.shape[0], q.shape[1]
        hkv = k.shape[1]
        nseq = 1 if cu is None else cu.numel() - 1
        timings = {}
        for unit in candidates:
            a = cls(T, hq, hkv, topk, nseq=nseq, unit=unit, **kw)
            o, lse = a.forward(q, k, v, idx, cu)
            a.backward(q, k, v, o, lse, do, cu)                      # warm-up
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                o, lse = a.forward(q, k, v, idx, cu)
                a.backward(q, k, v, o, lse, do, cu)
            e1.record()
            torch.cuda.synchronize()
            timings[unit] = e0.elapsed_time(e1) / reps
            del a
        best = min(timings, key=timings.get)
        return cls(T, hq, hkv, topk, nseq=nseq, unit=best, **kw), timings

    def build_index(self, idx, cu=None):
        build_index(self.shape, idx, cu, self.index_ws)

    def forward(self, q, k, v, idx, cu=None, rebuild_index=True, out=None, lse=None):
        s = self.shape
        o = torch.empty(s.total_tokens, s.hq, 128, dtype=torch.bfloat16, device=self.device) if out is None else out
        l = torch.empty(s.total_tokens, s.hq, dtype=torch.float32, device=self.device) if lse is None else lse
        nsa_sel_fwd(s, q, k, v, idx, cu, rebuild_index, self.index_ws, o, l, self.fwd_ws)
        return o, l

    def forward_static(self, q, k, v, idx, cu=None, rebuild_index=True, out=None, lse=None):
        """(O, LSE) by nsa_sel_fwd_static: the forward that keeps its partial results in the library's own device
        array instead of this object's workspace (small shapes only)."""
        s = self.shape
        o = torch.empty(s.total_tokens, s.hq, 128, dtype=torch.bfloat16, device=self.device) if out is None else out
        l = torch.empty(s.total_tokens, s.hq, dtype=torch.float32, device=self.device) if lse is None else lse
        nsa_sel_fwd_static(s, q, k, v, idx, cu, rebuild_index, self.index_ws, o, l)
        return o, l

    def backward(self, q, k, v, o, lse, do, cu=None, out=None):
        s = self.shape
        if out is None:
            dq = torch.empty_like(q)
            dk = torch.empty_like(k)
            dv = torch.empty_like(v)
        else:
            dq, dk, dv = out
        if self.bwd_ws is None:
            raise NsaSelError("this SelAttention was created with bwd=False")
        nsa_sel_bwd(s, q, k, v, o, lse, do, cu, self.index_ws, dq, dk, dv, self.bwd_ws)
        return dq, dk, dv

    def forward_query_outer(self, q, k, v, idx, cu=None):
        """(O, LSE) by the query-outer kernel (nsa_sel_fwd_query_outer): the loop order of the original NSA kernel."""
        s = self.shape
        o = torch.empty(s.total_tokens, s.hq, 128, dtype=torch.bfloat16, device=self.device)
        l = torch.empty(s.total_tokens, s.hq, dtype=torch.float32, device=self.device)
        expect_attention_args(s, self.device, q=q, k=k, v=v, idx=idx, cu=cu, need_idx=True)
        with torch.cuda.device(self.device):
            _check(lib().nsa_sel_fwd_query_outer(C.byref(s), _ptr(q), _ptr(k), _ptr(v), _ptr(idx), _ptr(cu), _ptr(o),
                                                 _ptr(l), _stream(self.device)), "nsa_sel_fwd_query_outer")
        return o, l

    def forward_gated(self, q, k, v, idx, gate, o_acc=None, cu=None, rebuild_index=True, out=None):
        """(O_out, O, LSE) with O_out = O_acc + gate * O (nsa_sel_fwd_gated); `out` may be the O_acc tensor."""
        s = self.shape
        o = torch.empty(s.total_tokens, s.hq, 128, dtype=torch.bfloat16, device=self.device)
        l = torch.empty(s.total_tokens, s.hq, dtype=torch.float32, device=self.device)
        o_out = torch.empty_like(o) if out is None else out
        expect_attention_args(s, self.device, q=q, k=k, v=v, idx=idx, cu=cu, gate=gate, o_acc=o_acc, o_out=o_out, o=o,
                              need_idx=bool(rebuild_index))
        with torch.cuda.device(self.device):
            _check(lib().nsa_sel_fwd_gated(C.byref(s), _ptr(q), _ptr(k), _ptr(v), _ptr(idx), _ptr(cu),
                                           int(rebuild_index), _ptr(self.index_ws), _nbytes(self.index_ws), _ptr(o),
                                           _ptr(l), _ptr(gate), _ptr(o_acc), _ptr(o_out), _ptr(self.fwd_ws),
                                           _nbytes(self.fwd_ws), _stream(self.device)), "nsa_sel_fwd_gated")
        return o_out, o, l

    def backward_gated(self, q, k, v, o, lse, do_out, gate, cu=None):
        """(dQ, dK, dV, dgate) of nsa_sel_bwd_gated."""
        s = self.shape
        dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        dgate = torch.empty(s.total_tokens, s.hq, dtype=torch.float32, device=self.device)
        expect_attention_args(s, self.device, q=q, k=k, v=v, cu=cu, o=o, lse=lse, do=do_out, gate=gate)
        if self.bwd_ws is None:
            raise NsaSelError("this SelAttention was created with bwd=False")
        with torch.cuda.device(self.device):
            _check(lib().nsa_sel_bwd_gated(C.byref(s), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(do_out),
                                           _ptr(gate), _ptr(cu), _ptr(self.index_ws), _nbytes(self.index_ws), _ptr(dq),
                                           _ptr(dk), _ptr(dv), _ptr(dgate), _ptr(self.bwd_ws), _nbytes(self.bwd_ws),
                                           _stream(self.device)), "nsa_sel_bwd_gated")
        return dq, dk, dv, dgate

    def dense_entries(self):
        """Boolean host array over the list entries (in list order): True where the forward routes the entry's
        (query tile, KV block) pair through the dense path (the sign bit of the entry's column)."""
        (o_cnt, o_off, o_qe, o_vm), bcap = index_view(self.shape, self.index_ws)
        nl = self.shape.hkv * bcap
        raw = self.index_ws
        npairs = int(raw[o_off + 4 * nl:o_off + 4 * nl + 4].view(torch.int32).item())
        qent = raw[o_qe:o_qe + 8 * npairs].view(torch.int32).cpu().numpy().reshape(npairs, 2)
        return qent[:, 1] < 0

    def index_arrays(self):
        """Host copies of (cnt [hkv, b_cap], off, qlist, qslot, vmask [T, hkv]) for inspection."""
        (o_cnt, o_off, o_qe, o_vm), bcap = index_view(self.shape, self.index_ws)
        s = self.shape
        nl = s.hkv * bcap
        raw = self.index_ws
        def ints(off, n):
            return raw[off:off + 4 * n].view(torch.int32).cpu().numpy()
        cnt = ints(o_cnt, nl).reshape(s.hkv, bcap)
        off = ints(o_off, nl + 1)
        npairs = int(off[-1])
        qent = ints(o_qe, 2 * npairs).reshape(npairs, 2)
        # the sign bit of an entry's column flags a dense (tile, block) pair (the forward's routing, not part of the
        # inversion result)
        return cnt, off, qent[:, 0].copy(), (qent[:, 1] & 0x7FFFFFFF).copy(), ints(o_vm, s.total_tokens * s.hkv).reshape(
            s.total_tokens, s.hkv).view("uint32"), bcap
