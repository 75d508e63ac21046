"""Host-side logic of the HIP library (split bounds, size and workspace arithmetic, argument
validation of the entry points) under AddressSanitizer and UndefinedBehaviorSanitizer.

The library's sources are compiled once more with the sanitizers on the host side only (device code
is built without them) and linked with a plain-C driver, ``tests/helpers/host_sanitize_main.c``,
whose calls all return before anything is enqueued on a GPU, so the program runs here without one."""

import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(ROOT, "paper_2204_06787_amd", "csrc")
SOURCES = ["marsit_fused.hip", "marsit_worker_ops.hip", "marsit_diagnostics.hip", "marsit_pipeline.hip"]
SANITIZE = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-gpu-sanitize", "-fno-omit-frame-pointer"]


def test_library_host_code_runs_clean_under_asan_and_ubsan(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    clang = "/opt/rocm/llvm/bin/clang"
    if not (os.path.exists(hipcc) and os.path.exists(clang)):
        pytest.skip("no hipcc / clang here")
    include = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    jobs = []
    for name in SOURCES:                                   # one compiler process per source, side by side
        obj = str(tmp_path / (name + ".o"))
        cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-std=c++17", "-ffp-contract=off",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", *SANITIZE, *include,
               "-c", os.path.join(CSRC, name), "-o", obj]
        jobs.append((obj, cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    objects = []
    for obj, cmd, proc in jobs:
        out, _ = proc.communicate(timeout=900)
        assert proc.returncode == 0, " ".join(cmd) + "\n" + out
        objects.append(obj)
    main_obj = str(tmp_path / "main.o")
    subprocess.run([clang, "-std=c11", "-O1", "-g", *[f for f in SANITIZE if f != "-fno-gpu-sanitize"], *include,
                    "-c", os.path.join(HERE, "helpers", "host_sanitize_main.c"), "-o", main_obj],
                   check=True, capture_output=True, text=True)
    exe = str(tmp_path / "host_sanitize")
    link = subprocess.run([hipcc, "-fsanitize=address,undefined", "-fno-gpu-sanitize", main_obj, *objects, "-o", exe],
                          capture_output=True, text=True)
    assert link.returncode == 0, link.stdout + link.stderr
    # leak detection is off: the HIP runtime keeps its own allocations until the process ends
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert run.stdout.strip().endswith("ok")
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr
