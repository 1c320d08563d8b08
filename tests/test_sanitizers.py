"""Sanitizer leg: the HIP-free host layer (chunk packer, scheduler, per-chunk metadata) and the C oracle, built
with gcc -fsanitize=address,undefined into one program (tests/sanitize_host.cpp) that drives them with heap
buffers of exactly the required size and checks the results against a token-stream re-derivation and closed
forms.  Any access past a capacity, misaligned access or signed overflow in their index arithmetic fails the run.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None or shutil.which("gcc") is None, reason="needs gcc / g++")
def test_host_layer_and_oracle_under_asan_ubsan(tmp_path):
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
    inc = ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2401_11181_amd", "csrc")]
    objs = []
    for compiler, src, extra in (
            ("gcc", os.path.join(ROOT, "oracle", "tetri_oracle.c"), ["-std=c11", "-fopenmp"]),
            ("g++", os.path.join(ROOT, "paper_2401_11181_amd", "csrc", "tetri_plan.cpp"), ["-std=c++17"]),
            ("g++", os.path.join(ROOT, "tests", "sanitize_host.cpp"), ["-std=c++17"])):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        subprocess.run([compiler, "-c", src, "-o", obj, "-Wall"] + extra + san + inc, check=True)
        objs.append(obj)
    exe = str(tmp_path / "sanitize_host")
    subprocess.run(["g++", "-o", exe] + objs + san + ["-static-libasan", "-static-libubsan", "-fopenmp"], check=True)
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    res = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "sanitize_host: ok" in res.stdout
