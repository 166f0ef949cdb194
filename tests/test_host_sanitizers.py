"""The host code of the library under AddressSanitizer and UndefinedBehaviorSanitizer, without a GPU.

Every source is compiled once more with both sanitizers on its host half only (device code is untouched), linked
with tests/host_sanitize_main.cpp, and run.  The driver calls each entry point in a way that ends on the host: size
and offset queries over a grid of configurations, every launching call stopped by its argument checks, and the
pipeline-degree routine (Sec. 4) on random models.  A sanitizer report or a failed expectation fails the test."""
import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

from paper_2501_10714_amd.build import CSRC, SOURCES

HERE = os.path.dirname(os.path.abspath(__file__))
CLANGXX = "/opt/rocm/lib/llvm/bin/clang++"
SAN = ["-fsanitize=address", "-fsanitize=undefined"]


@pytest.mark.skipif(shutil.which("hipcc") is None or not os.path.exists(CLANGXX), reason="needs the ROCm compilers")
def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    host_san = [a for s in SAN for a in ("-Xarch_host", s)]

    def compile_one(src):
        obj = str(tmp_path / src.replace(".hip", ".o"))
        cmd = ["hipcc", "--offload-arch=gfx950", "-O1", "-g0", "-std=c++17", "-fPIC", *host_san, "-Xclang", "-target-feature",
               "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-c", os.path.join(CSRC, src), "-o", obj]
        p = subprocess.run(cmd, capture_output=True, text=True)
        assert p.returncode == 0, f"{src}:\n{p.stderr[-3000:]}"
        return obj

    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    main_o = str(tmp_path / "main.o")
    subprocess.run([CLANGXX, "-std=c++17", "-O1", "-g", *SAN, "-fno-sanitize-recover=undefined", "-c",
                    os.path.join(HERE, "host_sanitize_main.cpp"), "-o", main_o], check=True)
    exe = str(tmp_path / "host_san")
    subprocess.run([CLANGXX, *SAN, main_o, *objs, "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib", "-o", exe],
                   check=True)
    # the HIP runtime keeps its own allocations until the process ends: leaks are not what this test is about
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    p = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert p.returncode == 0 and "host sanitizer driver: ok" in p.stdout, p.stdout[-3000:] + p.stderr[-3000:]
    assert "runtime error" not in p.stderr and "AddressSanitizer" not in p.stderr, p.stderr[-3000:]
