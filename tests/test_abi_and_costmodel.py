"""Host-side checks that need no GPU: the C ABI exports what the header declares, argument validation, and the
paper's cost model against the two ratios the paper prints."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _lib():
    import paper_2508_18224_amd as nsa
    return nsa, nsa.lib()


def test_library_exports_every_declared_symbol():
    nsa, L = _lib()
    header = open(os.path.join(ROOT, "include", "nsa_sel.h")).read()
    declared = set(re.findall(r"\b(nsa_sel_[a-z_]+)\s*\(", header))
    assert declared == set(nsa.SYMBOLS)
    for name in declared:
        assert hasattr(L, name), name


def test_measuring_build_exports_the_same_boundary_plus_its_reader():
    """libnsa_sel_timing.so (cycle stamps in the pipelined backward, see pipe_timing.py) is the same library otherwise."""
    import ctypes
    from paper_2508_18224_amd.build import LIB_TIMING
    nsa, _ = _lib()
    assert os.path.exists(LIB_TIMING), "python -m paper_2508_18224_amd.build builds it"
    T = ctypes.CDLL(LIB_TIMING)
    for name in nsa.SYMBOLS + ["nsa_sel_pipe_timing_read"]:
        assert hasattr(T, name), name


def test_shape_validation_happens_on_the_host():
    nsa, L = _lib()
    ok = nsa.Shape(4096, 1, 8, 2, 128, 64, 16, 1, 0.0, 0)
    gather_only = nsa.Shape(4096, 1, 8, 2, 128, 64, 16, 1, 0.0, 0, 0, 0, -1)     # dense path off
    f, b, i = nsa.workspace_bytes(gather_only)
    assert f >= 4096 * 8 * 16 * 128 * 2 and b > f and i > 0
    assert nsa.workspace_bytes(nsa.Shape(4096, 1, 8, 2, 128, 128, 8, 1, 0.0, 0, 0, 0, -1))[0] * 2 == f   # half the slots
    fmin, bmin = nsa.workspace_bytes_min(gather_only)        # one of the two KV heads per pass
    assert fmin * 2 == f and fmin >= 4096 * 4 * 16 * 128 * 2 and fmin < bmin < b
    assert nsa.workspace_bytes(ok) == (f, b, i)              # the dense route needs no workspace of its own
    bad = [
        (nsa.Shape(4096, 1, 8, 3, 128, 64, 16, 1, 0.0, 0), -1),     # hq % hkv
        (nsa.Shape(4096, 1, 18, 2, 128, 64, 16, 1, 0.0, 0), -1),    # g = 9
        (nsa.Shape(4096, 0, 8, 2, 128, 64, 16, 1, 0.0, 0), -1),     # nseq
        (nsa.Shape(4096, 1, 8, 2, 64, 64, 16, 1, 0.0, 0), -2),      # d
        (nsa.Shape(4096, 1, 8, 2, 128, 256, 16, 1, 0.0, 0), -2),    # block
        (nsa.Shape(4096, 1, 8, 2, 128, 128, 33, 1, 0.0, 0), -2),    # topk
        (nsa.Shape(4096, 1, 8, 2, 128, 64, 33, 1, 0.0, 0), -2),     # topk
        (nsa.Shape(2 ** 30, 1, 8, 2, 128, 64, 16, 1, 0.0, 0), -2),  # too large
        (nsa.Shape(4096, 1, 8, 2, 128, 64, 16, 1, 0.0, 0, -5), -1),   # negative window
        (nsa.Shape(4096, 1, 8, 2, 128, 64, 16, 0, 0.0, 0, 512), -1),  # window without causal
        (nsa.Shape(4096, 1, 8, 2, 128, 64, 16, 1, 0.0, 0, 0, 300), -1),   # unit not a power of two
        (nsa.Shape(4096, 1, 8, 2, 128, 64, 16, 1, 0.0, 0, 0, 4096), -1),  # unit too large
        (nsa.Shape(4096, 1, 8, 2, 128, 64, 16, 1, 0.0, 0, 0, 0, 2), -1),     # dense outside [-1, 1]
    ]
    sz = ctypes.c_size_t()
    for shape, code in bad:
        assert L.nsa_sel_workspace_bytes(ctypes.byref(shape), ctypes.byref(sz), None, None) == code
    # null pointers are rejected before anything is launched (no GPU is touched)
    assert L.nsa_sel_build_index(ctypes.byref(ok), None, None, None, 0, None) == -1
    assert L.nsa_sel_fwd(ctypes.byref(ok), None, None, None, None, None, 1, None, 0, None, None, None, 0, None) == -1
    # a misaligned tensor pointer is an argument error, found before any size check or launch
    vp = ctypes.c_void_p
    assert L.nsa_sel_fwd(ctypes.byref(ok), vp(4096 + 2), vp(4096), vp(4096), None, None, 0, vp(4096), 1 << 40, vp(4096),
                         vp(4096), vp(4096), 1 << 40, None) == -1
    assert b"workspace" in L.nsa_sel_strerror(-3)


def test_paper_cost_ratios():
    from paper_2508_18224_amd import cost_model as cm
    rows = [l.split() for l in open(os.path.join(ROOT, "tests", "golden", "paper_cost_ratios.txt"))
            if l.strip() and not l.startswith("#")]
    for g, B_K, T, mem_pct, flop_pct in rows:
        g, B_K, T = int(g), int(B_K), int(T)
        N, h_K, d = 65536, 8, 128
        h = g * h_K
        mem = cm.fsa_total_bytes(N, h, h_K, d, T) / cm.nsa_bytes(N, h, h_K, d, B_K, T)
        fl = cm.fsa_total_flops(N, h, h_K, d, B_K, T) / cm.nsa_flops(N, h_K, d, B_K, T)
        assert abs(100 * mem - float(mem_pct)) < 0.06
        assert abs(100 * fl - float(flop_pct)) < 0.06
    f, b = cm.effective_flops(65536, 32, 16)
    assert f == 4.0 * 65536 * 32 * 16 * 64 * 128 and b == 2.5 * f


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2508_18224_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, fn)).read()
                assert "oracle" not in text, fn


def test_binding_validates_tensors_on_the_host():
    """dtype, shape, device and contiguity of every tensor are checked before an address reaches the library."""
    import torch
    nsa, _ = _lib()
    from paper_2508_18224_amd import binding as B
    s = nsa.Shape(256, 2, 8, 2, 128, 64, 4, 1, 0.0, 0)
    bf, f32, i32 = torch.bfloat16, torch.float32, torch.int32
    good = dict(q=torch.zeros(256, 8, 128, dtype=bf), k=torch.zeros(256, 2, 128, dtype=bf),
                v=torch.zeros(256, 2, 128, dtype=bf), idx=torch.zeros(256, 2, 4, dtype=i32),
                cu=torch.tensor([0, 100, 256], dtype=i32), o=torch.zeros(256, 8, 128, dtype=bf),
                lse=torch.zeros(256, 8, dtype=f32), do=torch.zeros(256, 8, 128, dtype=bf),
                gate=torch.zeros(256, 8, dtype=f32))
    B.expect_attention_args(s, "cpu", need_idx=True, **good)                 # all consistent: passes
    bad = {
        "q": [good["q"].float(), good["q"].half(), good["q"][:255], good["q"].transpose(0, 1).contiguous()],
        "k": [good["k"].float(), torch.zeros(256, 8, 128, dtype=bf)],
        "idx": [good["idx"].long(), torch.zeros(256, 2, 16, dtype=i32), None],
        "cu": [good["cu"].long(), torch.tensor([0, 256], dtype=i32), None],
        "lse": [good["lse"].double(), torch.zeros(256, 2, dtype=f32)],
        "gate": [good["gate"].double(), torch.zeros(256, dtype=f32)],
        "do": [good["do"].float(), torch.zeros(128, 8, 128, dtype=bf)],
    }
    for name, cases in bad.items():
        for t in cases:
            with pytest.raises(nsa.NsaSelError):
                B.expect_attention_args(s, "cpu", need_idx=True, **{**good, name: t})
    with pytest.raises(nsa.NsaSelError):                                  # a strided view
        B.expect_attention_args(s, "cpu", **{**good, "q": torch.zeros(256, 8, 256, dtype=bf)[:, :, ::2]})
    with pytest.raises(nsa.NsaSelError):                                  # wrong device
        B.expect_attention_args(s, "cuda:0", **good)
    with pytest.raises(nsa.NsaSelError):                                  # the gated sum may not alias O
        B.expect_attention_args(s, "cpu", **{**good, "o_acc": good["o"]})
    with pytest.raises(nsa.NsaSelError):
        B.expect_attention_args(s, "cpu", **{**good, "o_out": good["o"]})
    with pytest.raises(nsa.NsaSelError):                                  # gradients: dk with query-head count
        B.expect_attention_args(s, "cpu", grads=(good["q"], good["q"], good["k"]), **good)
    # workspaces are sized in bytes whatever the element type of the tensor that holds them
    need = nsa.workspace_bytes_min(s)[0]
    B.expect_workspace("ws", torch.zeros((need + 3) // 4, dtype=torch.float32), need, "cpu")
    with pytest.raises(nsa.NsaSelError):
        B.expect_workspace("ws", torch.zeros(need // 4 - 1, dtype=torch.float32), need, "cpu")
    with pytest.raises(nsa.NsaSelError):
        B.expect_workspace("ws", torch.zeros(need, dtype=torch.uint8), need, "cuda:0")
    # the entry points run these checks before they touch the library: a CPU tensor never reaches a kernel
    ws = torch.zeros(16, dtype=torch.uint8)
    with pytest.raises(nsa.NsaSelError):
        nsa.nsa_sel_fwd(s, good["q"], good["k"], good["v"], good["idx"], good["cu"], True, ws, good["o"], good["lse"], ws)


def test_gated_forward_rejects_aliasing_of_the_ungated_output():
    nsa, L = _lib()
    ok = nsa.Shape(4096, 1, 8, 2, 128, 64, 16, 1, 0.0, 0)
    vp = ctypes.c_void_p
    a, b, c = vp(4096), vp(8192), vp(16384)
    big = 1 << 40
    # O_out == O and O_acc == O are argument errors, found on the host before any launch
    assert L.nsa_sel_fwd_gated(ctypes.byref(ok), a, a, a, a, None, 0, a, big, b, a, a, None, b, a, big, None) == -1
    assert L.nsa_sel_fwd_gated(ctypes.byref(ok), a, a, a, a, None, 0, a, big, b, a, a, b, c, a, big, None) == -1


def test_static_forward_refuses_large_shapes_before_any_gpu_call():
    nsa, L = _lib()
    vp = ctypes.c_void_p
    a = vp(4096)
    fits = nsa.Shape(4032, 1, 32, 8, 128, 64, 16, 1, 0.0, 0)       # one KV head: 4032 * 4 * 16 * 260 B < 64 MiB
    big = nsa.Shape(4096, 1, 32, 8, 128, 64, 16, 1, 0.0, 0)
    assert nsa.workspace_bytes_min(fits)[0] <= 64 << 20 < nsa.workspace_bytes_min(big)[0]
    assert L.nsa_sel_fwd_static(ctypes.byref(big), a, a, a, a, None, 1, a, 1 << 40, a, a, None) == -5
    assert b"nsa_sel_fwd_static" in L.nsa_sel_strerror(-5)
    assert L.nsa_sel_fwd_static(ctypes.byref(fits), None, a, a, a, None, 1, a, 1 << 40, a, a, None) == -1
    assert L.nsa_sel_fwd_static(ctypes.byref(fits), a, a, a, a, None, 1, a, 16, a, a, None) == -3
