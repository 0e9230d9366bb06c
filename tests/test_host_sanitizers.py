"""The boundary's host code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU).

The library's host side -- argument checks, the MDS check of the generators, block geometry, the
error paths of codenet_encode that release a half-built layer -- is compiled with
`-Xarch_host -fsanitize=address -Xarch_host -fsanitize=undefined` (device code is not instrumented)
into a scratch directory, linked into tests/host/boundary_driver.cpp, and run.  Without a device every
allocation fails, which is exactly the path that has to clean up after itself."""
import os
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_1903_01042_amd", "csrc")
HIPCC = "/opt/rocm/bin/hipcc"
CLANGXX = "/opt/rocm/lib/llvm/bin/clang++"
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
       "-Xarch_host", "-fno-sanitize-recover=undefined"]


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="no hipcc")
def test_boundary_error_paths_are_clean_under_the_sanitizers():
    tmp = tempfile.mkdtemp(prefix="codenet_asan_")
    try:
        flags = ["--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
                 "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                 "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-Wno-unused-command-line-argument"] + SAN
        procs = []
        for src in ("api", "gemm", "gemm_bf16", "kernels"):
            procs.append(subprocess.Popen([HIPCC] + flags + ["-c", os.path.join(CSRC, src + ".hip"), "-o",
                                                            os.path.join(tmp, src + ".o")],
                                          stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True))
        for p in procs:
            out, _ = p.communicate(timeout=600)
            assert p.returncode == 0, out[-3000:]
        exe = os.path.join(tmp, "boundary_driver")
        drv = os.path.join(tmp, "boundary_driver.o")
        res = subprocess.run([CLANGXX, "-std=c++17", "-O1", "-g", "-fsanitize=address", "-fsanitize=undefined",
                              "-fno-sanitize-recover=undefined", "-I" + os.path.join(ROOT, "include"), "-c",
                              os.path.join(ROOT, "tests", "host", "boundary_driver.cpp"), "-o", drv],
                             capture_output=True, text=True, timeout=600)
        assert res.returncode == 0, res.stderr[-3000:]
        link = [HIPCC, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", drv]
        link += [os.path.join(tmp, s + ".o") for s in ("api", "gemm", "gemm_bf16", "kernels")] + ["-o", exe]
        res = subprocess.run(link, capture_output=True, text=True, timeout=600)
        assert res.returncode == 0, res.stderr[-3000:]
        env = dict(os.environ)
        env["ASAN_OPTIONS"] = "detect_leaks=1:verify_asan_link_order=0:halt_on_error=1"
        env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
        run = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
        report = run.stdout[-3000:] + run.stderr[-3000:]
        assert run.returncode == 0, report
        assert "all checks passed" in run.stdout, report
        assert "ERROR: AddressSanitizer" not in run.stderr and "runtime error" not in run.stderr, report
        assert "LeakSanitizer" not in run.stderr, report
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
