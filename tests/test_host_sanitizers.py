"""The library's host code under AddressSanitizer and UndefinedBehaviorSanitizer.  Every source is compiled at -O1
(seconds per file) with both sanitizers on the host side and linked with tests/host_checks/abi_host_checks.cpp
into one program that walks the host-side paths of the C-ABI (validation, layout arithmetic at extreme field values,
creation, calls out of order, tables).  The sanitizers' runtime is linked into the program itself, so nothing is
preloaded; kernels are never launched."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2407_02328_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
       "-Xarch_host", "-fno-sanitize-recover=undefined"]


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="no hipcc")
def test_host_paths_are_clean_under_asan_and_ubsan(tmp_path):
    from paper_2407_02328_amd.build import SOURCES
    objs = []
    procs = []
    for src in SOURCES:
        obj = str(tmp_path / (os.path.splitext(src)[0] + ".o"))
        objs.append(obj)
        procs.append(subprocess.Popen(
            [HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             *SAN, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c", os.path.join(CSRC, src), "-o", obj],
            stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True))
    for src, p in zip(SOURCES, procs):
        out, _ = p.communicate(timeout=600)
        assert p.returncode == 0, f"{src}:\n{out[-4000:]}"
    main_obj = str(tmp_path / "abi_host_checks.o")
    cc = subprocess.run(
        [HIPCC, "--offload-arch=gfx950", "--cuda-host-only", "-O1", "-g", "-std=c++17", *SAN,
         "-I", os.path.join(ROOT, "include"), "-c", os.path.join(ROOT, "tests", "host_checks", "abi_host_checks.cpp"),
         "-o", main_obj], capture_output=True, text=True, timeout=600)
    assert cc.returncode == 0, cc.stdout[-4000:] + cc.stderr[-4000:]
    exe = str(tmp_path / "abi_host_checks")
    link = subprocess.run([HIPCC, "--offload-arch=gfx950", *SAN, main_obj, *objs, "-o", exe],
                          capture_output=True, text=True, timeout=600)
    assert link.returncode == 0, link.stdout[-4000:] + link.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    report = run.stdout[-3000:] + run.stderr[-6000:]
    assert run.returncode == 0 and "host checks ok" in run.stdout, report
    assert "Sanitizer" not in run.stderr and "runtime error" not in run.stderr, report
