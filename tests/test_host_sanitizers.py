"""The host side of the library (header parsing, the memory plan, every error path that returns before device
work) under AddressSanitizer and UndefinedBehaviorSanitizer: tests/host_checks.cpp is linked against a copy of
the runtime translation unit whose HOST code is instrumented (the kernels' translation units come as they are
built for the library), and run here, without a GPU."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_code_under_asan_and_ubsan(tmp_path):
    from paper_2010_13887_amd import build as B
    if not all(os.path.exists(os.path.join(B.OBJ_DIR, os.path.splitext(s)[0] + ".o")) for s in B.SOURCES):
        B.build(verbose=False)
    hipcc = B._hipcc()
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
    rt = str(tmp_path / "lsq_runtime_san.o")
    r = subprocess.run([hipcc, *B.FLAGS, *san, "-g", "-c", os.path.join(B.CSRC, "lsq_runtime.hip"), "-o", rt],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    others = [os.path.join(B.OBJ_DIR, os.path.splitext(s)[0] + ".o") for s in B.SOURCES if s != "lsq_runtime.hip"]
    exe = str(tmp_path / "host_checks")
    clang = "/opt/rocm/lib/llvm/bin/clang++"
    main_o = str(tmp_path / "host_checks.o")
    host_san = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"]
    r = subprocess.run([clang, "-O1", "-g", "-std=c++17", *host_san, "-c", os.path.join(ROOT, "tests", "host_checks.cpp"),
                        "-o", main_o], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "--hip-link", *host_san, main_o, rt, *others, "-o", exe],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    # whatever the environment preloads stays preloaded: the runtime's check of its place in the library list is switched off
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0 and "all passed" in r.stdout, (r.stdout[-2000:], r.stderr[-3000:])
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-3000:]
