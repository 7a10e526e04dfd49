"""Host code of the library under AddressSanitizer + UndefinedBehaviorSanitizer (no GPU).

The four host sources are compiled with clang's sanitizers together with stand-ins for the kernel
launchers (tests/capi/launch_stubs.cpp) and a C fuzz driver (tests/capi/host_fuzz.c) that pushes
3000 random nets through planning, plan read-back, options, tile-table layout, workspace sizing,
the refusal of launches on an unbound plan, the scaling curve and the cost fit.  Any sanitizer
report or unexpected return code fails the test."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANG = "/opt/rocm/lib/llvm/bin/clang"


@pytest.mark.skipif(not os.path.exists(CLANG), reason="ROCm clang not found")
def test_host_entry_points_are_clean_under_asan_and_ubsan(tmp_path):
    csrc = os.path.join(ROOT, "paper_1811_11141_amd", "csrc")
    # plain host C/C++ only; -fno-gpu-sanitize states that no device code is instrumented
    san = ["-fsanitize=address,undefined", "-fno-gpu-sanitize", "-Wno-unused-command-line-argument",
           "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
    objs = []
    for src in ("api.cpp", "planner.cpp", "tables.cpp", "executor.cpp"):
        obj = str(tmp_path / (src + ".o"))
        cmd = [CLANG + "++", "-std=c++17", "-c", *san, "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
               "-ffp-contract=off", os.path.join(csrc, src), "-o", obj]
        res = subprocess.run(cmd, capture_output=True, text=True)
        assert res.returncode == 0, res.stderr[-3000:]
        objs.append(obj)
    stub = str(tmp_path / "stubs.o")
    res = subprocess.run([CLANG + "++", "-std=c++17", "-c", *san, "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
                          os.path.join(ROOT, "tests", "capi", "launch_stubs.cpp"), "-o", stub],
                         capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-3000:]
    drv = str(tmp_path / "fuzz.o")
    res = subprocess.run([CLANG, "-std=c99", "-c", *san, "-I", os.path.join(ROOT, "include"),
                          os.path.join(ROOT, "tests", "capi", "host_fuzz.c"), "-o", drv], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-3000:]
    exe = str(tmp_path / "host_fuzz")
    res = subprocess.run([CLANG + "++", *san, drv, stub, *objs, "-o", exe, "-L/opt/rocm/lib", "-lamdhip64",
                          "-Wl,-rpath,/opt/rocm/lib"], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:protect_shadow_gap=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-4000:])
    assert "done, bad = 0" in run.stdout
    assert "ERROR" not in run.stderr and "runtime error" not in run.stderr, run.stderr[-4000:]
