"""Address- and undefined-behaviour-sanitizer run of the host code that indexes memory by hand:
the oracle's C routines and the library's packing and native tiling (CPU only; the GPU code
cannot run under these sanitizers)."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_and_host_packing_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "sanitize_driver")
    san = ["-fsanitize=address,undefined", "-static-libasan", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
    obj = str(tmp_path / "rb_oracle.o")
    subprocess.check_call(["gcc", "-std=c11", "-Wall", "-Wextra", *san, "-c",
                           os.path.join(ROOT, "oracle", "rb_oracle.c"), "-o", obj])
    subprocess.check_call(["g++", "-std=c++17", "-Wall", *san,
                           "-I", os.path.join(ROOT, "include"),
                           "-I", os.path.join(ROOT, "paper_2602_05367_amd", "csrc"),
                           os.path.join(ROOT, "tests", "sanitize", "driver.cpp"),
                           os.path.join(ROOT, "paper_2602_05367_amd", "csrc", "rb_host.cpp"),
                           obj, "-o", exe])
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0"
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=120)
    assert res.returncode == 0, res.stdout
    assert "all shapes passed" in res.stdout
    assert "runtime error" not in res.stdout and "AddressSanitizer" not in res.stdout, res.stdout
