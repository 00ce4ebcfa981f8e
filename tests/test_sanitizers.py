"""CPU-only sanitizer runs: the oracle, and the host side of the library's entry points
(argument validation, work plan, workspace sizing), each built with
-fsanitize=address,undefined into a small program of its own and run here.  Nothing is
launched on a GPU."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:halt_on_error=1",
           UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def run(cmd, **kw):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert res.returncode == 0, " ".join(cmd) + "\n" + res.stdout[-4000:]
    return res.stdout


def test_oracle_runs_clean_under_address_and_undefined_sanitizers(tmp_path):
    src = [os.path.join(ROOT, "oracle", "ts_oracle.c"), os.path.join(SAN, "oracle_driver.c")]
    san, plain = str(tmp_path / "oracle_san"), str(tmp_path / "oracle_plain")
    run(["gcc", "-std=c99", "-g", "-O1", "-fno-omit-frame-pointer", "-fopenmp",
         "-fsanitize=address,undefined", "-fno-sanitize-recover=all"] + src + ["-o", san, "-lm"])
    run(["gcc", "-std=c99", "-O2", "-fopenmp"] + src + ["-o", plain, "-lm"])
    out_san = run([san], env=ENV)
    out_plain = run([plain])
    assert out_san.strip().endswith("ok")
    assert out_san == out_plain, "the sanitized and the plain build of the oracle disagree"


def test_host_side_of_the_entry_points_runs_clean_under_sanitizers(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    csrc = os.path.join(ROOT, "paper_2509_12211_amd", "csrc")
    inc = os.path.join(ROOT, "include")
    host_san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer"]
    common = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC",
              "-Wno-unknown-warning-option", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
    objs = []
    for name, path in (("entry", os.path.join(csrc, "tinyserve.hip")),
                       ("stubs", os.path.join(SAN, "format_stubs.hip"))):
        obj = str(tmp_path / (name + ".o"))
        run(common + host_san + ["-I", csrc, "-c", path, "-o", obj])
        objs.append(obj)
    drv = str(tmp_path / "driver.o")
    run(common + host_san + ["-I", inc, "-x", "hip", "-c", os.path.join(SAN, "abi_driver.cpp"), "-o", drv])
    exe = str(tmp_path / "abi_san")
    run([hipcc, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize"]
        + objs + [drv, "-o", exe])
    out = run([exe], env=dict(ENV, ASAN_OPTIONS=ENV["ASAN_OPTIONS"].replace("detect_leaks=1", "detect_leaks=0")))
    assert out.strip().endswith("ok"), out
