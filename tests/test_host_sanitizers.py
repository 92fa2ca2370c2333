"""The library's host side (argument validation, capacity and workspace arithmetic, contexts) under AddressSanitizer and
UndefinedBehaviorSanitizer: every source is compiled with the sanitizers on the host pass only, linked with a driver that
makes valid and invalid calls under a dry-run context (no GPU needed), with every structure the library reads in a heap
block of exactly its size."""
import glob
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
CLANGXX = "/opt/rocm/llvm/bin/clang++"
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all"]


@pytest.mark.skipif(not (os.path.exists(HIPCC) and os.path.exists(CLANGXX)), reason="needs hipcc and its clang++")
def test_host_side_under_asan_and_ubsan(tmp_path):
    objs, procs = [], []
    for src in sorted(glob.glob(os.path.join(ROOT, "paper_2504_18082_amd", "csrc", "*.hip"))):
        obj = str(tmp_path / (os.path.basename(src)[:-4] + ".o"))
        objs.append(obj)
        cmd = [HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"] + SAN
        procs.append(subprocess.Popen(cmd + ["-c", src, "-o", obj], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True))
    for p in procs:
        out, _ = p.communicate()
        assert p.returncode == 0, out
    drv = str(tmp_path / "driver.o")
    build = subprocess.run([CLANGXX, "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-c",
                            os.path.join(ROOT, "tests", "host_sanitize_driver.cpp"), "-o", drv], capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    exe = str(tmp_path / "host_sanitized")
    link = subprocess.run([HIPCC, "--offload-arch=gfx950", "-fsanitize=address,undefined", "-fno-gpu-sanitize", drv] + objs + ["-o", exe],
                          capture_output=True, text=True)
    assert link.returncode == 0, link.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0")        # (the HIP runtime's own start-up allocations are not ours to judge)
    run = subprocess.run([exe], capture_output=True, text=True, timeout=120, env=env)
    assert run.returncode == 0, run.stdout + run.stderr
    assert run.stdout.strip().endswith("ok")
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr
    shutil.rmtree(tmp_path, ignore_errors=True)
