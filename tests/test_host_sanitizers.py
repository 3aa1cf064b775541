"""The host side of the launcher under AddressSanitizer and UndefinedBehaviorSanitizer: api.hip and group.hip (argument
checks, the workspace plan) are compiled with the sanitizers on their host code only, linked with the ordinary
objects of the other sources into a small program that drives every error path of the C ABI (tests/host_sanitize/
abi_errors.cpp).  No GPU is touched: the checks reject every call before a launch."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_abi_error_paths_are_clean_under_asan_and_ubsan(tmp_path):
    from paper_2411_08446_amd import build
    others = ["hash", "centroid", "restore", "backward"]
    if not all(os.path.exists(os.path.join(build.BUILD_DIR, o + ".o")) for o in others):
        build.build(verbose=False)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined"]
    common = [build.HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-Wno-inline-asm",
              "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
    objs = []
    for src in (os.path.join(build.CSRC, "api.hip"), os.path.join(build.CSRC, "group.hip"),
                os.path.join(ROOT, "tests", "host_sanitize", "abi_errors.cpp")):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        res = subprocess.run(common + san + ["-c", src, "-o", obj], capture_output=True, text=True, timeout=600)
        assert res.returncode == 0, res.stderr
        objs.append(obj)
    exe = str(tmp_path / "abi_errors_san")
    link = [build.HIPCC, "--offload-arch=gfx950", *san, *objs, *[os.path.join(build.BUILD_DIR, o + ".o") for o in others], "-o", exe]
    res = subprocess.run(link, capture_output=True, text=True, timeout=600)
    assert res.returncode == 0, res.stderr
    res = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "0 failures" in res.stdout
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr
