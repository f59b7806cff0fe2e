"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the host code, run on the CPU: the C
oracle on small exact-size buffers, and the library's entry points on every validation path
(no GPU is touched: each call is rejected, or is an empty problem, before a kernel would be
enqueued).  The sanitizer runtimes are linked statically, so nothing has to be preloaded."""
import os
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2511_02647_amd", "csrc")
HIPCC = "/opt/rocm/bin/hipcc"
CLANGXX = "/opt/rocm/lib/llvm/bin/clang++"
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]


def run_clean(exe, env_extra):
    env = dict(os.environ, **env_extra)
    p = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=120)
    assert p.returncode == 0 and "clean" in p.stdout and "ERROR" not in p.stdout and "runtime error" not in p.stdout, p.stdout


def test_oracle_under_asan_and_ubsan():
    if shutil.which("gcc") is None:
        pytest.skip("gcc not found")
    with tempfile.TemporaryDirectory() as d:
        exe = os.path.join(d, "oracle_driver")
        subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-static-libasan"] + SAN +
                              ["-o", exe, os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"),
                               os.path.join(ROOT, "oracle", "fedattn_oracle.c"), "-lm"])
        run_clean(exe, {"ASAN_OPTIONS": "detect_leaks=1:abort_on_error=0", "OMP_NUM_THREADS": "4"})


def test_library_validation_paths_under_asan_and_ubsan():
    if not (os.path.exists(HIPCC) and os.path.exists(CLANGXX)):
        pytest.skip("ROCm compilers not found")
    host_san = [x for f in SAN for x in ("-Xarch_host", f)]
    flags = ["--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fno-gpu-rdc", "-w", "-Wno-inline-asm",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]
    with tempfile.TemporaryDirectory() as d:
        procs, objs = [], []
        for src in sorted(f for f in os.listdir(CSRC) if f.endswith(".hip")):
            obj = os.path.join(d, src.replace(".hip", ".o"))
            objs.append(obj)
            procs.append((src, subprocess.Popen([HIPCC] + flags + host_san + ["-c", os.path.join(CSRC, src), "-o", obj],
                                                stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        drv = os.path.join(d, "api_driver.o")
        subprocess.check_call([CLANGXX, "-std=c++17", "-O1", "-g"] + SAN + ["-I" + os.path.join(ROOT, "include"), "-c",
                               os.path.join(ROOT, "tests", "sanitize", "api_driver.cpp"), "-o", drv])
        for src, p in procs:
            out, _ = p.communicate()
            assert p.returncode == 0, "hipcc failed on %s:\n%s" % (src, out)
        exe = os.path.join(d, "api_driver")
        link = subprocess.run([HIPCC, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
                               "-static-libsan", "-o", exe, drv] + objs, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert link.returncode == 0, link.stdout
        # the HIP runtime keeps its own allocations until the process ends: no leak report for this one
        run_clean(exe, {"ASAN_OPTIONS": "detect_leaks=0:abort_on_error=0"})
