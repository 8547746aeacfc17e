"""The library's HOST code (argument validation, workspace layout arithmetic, error paths) under AddressSanitizer and
UndefinedBehaviorSanitizer: a sanitizer build of the library (device code unchanged, host pass instrumented) driven by a
small C program over ~10^4 shapes, no GPU involved.  GPU-side sanitizers are not available on this machine."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(not os.path.exists(HIPCC) or shutil.which("gcc") is None, reason="needs hipcc and gcc")
def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    from paper_2508_18224_amd.build import FLAGS, SOURCES
    lib = tmp_path / "libnsa_sel_san.so"
    src = [os.path.join(ROOT, "paper_2508_18224_amd", "csrc", s) for s in SOURCES]
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    res = subprocess.run([HIPCC, *FLAGS, *san, "-shared-libsan", "-o", str(lib), *src], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-3000:]
    exe = tmp_path / "host_abi_sanitize"
    clang = os.path.join(os.path.dirname(os.path.realpath(HIPCC)), "..", "lib", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/lib/llvm/bin/clang"
    res = subprocess.run([clang, "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-shared-libsan",
                          os.path.join(ROOT, "tests", "host_abi_sanitize.c"), "-o", str(exe), str(lib),
                          f"-Wl,-rpath,{tmp_path}"], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    # the sanitizer runtime of the toolchain that built the library
    rt = subprocess.run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True).stdout.strip()
    if rt and os.path.exists(rt):
        env["LD_LIBRARY_PATH"] = os.path.dirname(rt) + ":" + env.get("LD_LIBRARY_PATH", "")
    run = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=600)
    assert run.returncode == 0, (run.stdout + run.stderr)[-4000:]
    assert run.stdout.startswith("ok "), run.stdout
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr[-4000:]
