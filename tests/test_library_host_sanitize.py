"""The library's host logic under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU).

csrc/sparseloco.hip is compiled with the sanitizers on its HOST pass only (-Xarch_host; the device code is built as
usual and never runs here) together with tests/library_host_sanitize_main.cpp, which asks sparseloco_chunk_table
for the chunk tables -- the plan builder's own code: chunk geometry, strips, launch order -- of 400 seeded random
tensor lists in both layouts (empty tensors, vectors, narrow and wide matrices).  Every sanitizer report is fatal;
the driver also checks that every entry is a permutation member, that its present elements number n_c and that each
of them lies inside its tensor."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(not (os.path.exists(HIPCC) or shutil.which("hipcc")), reason="hipcc not found")
def test_plan_builder_under_sanitizers(tmp_path):
    exe = str(tmp_path / "library_host_sanitize")
    host = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]
    cmd = [HIPCC if os.path.exists(HIPCC) else "hipcc", "-O1", "-g", "-std=c++17", "--offload-arch=gfx950",
           "-ffp-contract=off", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
    for flag in host:
        cmd += ["-Xarch_host", flag]
    cmd += ["-I", os.path.join(ROOT, "include"),
            os.path.join(ROOT, "paper_2601_02360_amd", "csrc", "sparseloco.hip"),
            os.path.join(ROOT, "tests", "library_host_sanitize_main.cpp"),
            "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", "-o", exe]
    subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.PIPE)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=1", UBSAN_OPTIONS="halt_on_error=1")
    out = subprocess.run([exe], env=env, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=300)
    assert out.returncode == 0, out.stdout + out.stderr
    assert out.stdout.startswith("ok:"), out.stdout
