"""AddressSanitizer + UndefinedBehaviorSanitizer over the CPU side of the repository: the oracle's C routines on small
ragged inputs, and the host logic of the HIP library (validation, layouts, workspace sizes, argument checks) in a build
whose host code is instrumented.  Both are stand-alone executables, so nothing is preloaded into the test runner."""
import glob
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")


def _run(cmd, **kw):
    return subprocess.run(cmd, capture_output=True, text=True, timeout=900, **kw)


@pytest.mark.skipif(shutil.which("gcc") is None, reason="no gcc")
def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    res = _run(["gcc", "-O1", "-g", "-ffp-contract=off", "-fopenmp", "-std=c11", "-fsanitize=address,undefined",
                "-fno-sanitize-recover=undefined", "-o", exe, os.path.join(SAN, "oracle_driver.c"), "-lm"])
    assert res.returncode == 0, res.stderr[-3000:]
    run = _run([exe], env=dict(os.environ, ASAN_OPTIONS="detect_leaks=1", OMP_NUM_THREADS="4"))
    assert run.returncode == 0 and "oracle sanitizer run ok" in run.stdout, run.stdout[-2000:] + run.stderr[-4000:]
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="no hipcc")
def test_host_logic_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    from concurrent.futures import ThreadPoolExecutor

    src = sorted(glob.glob(os.path.join(ROOT, "paper_2102_04782_amd", "csrc", "*.hip")))
    inc = ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2102_04782_amd", "csrc")]
    # the host pass of every translation unit is instrumented (the flags sit behind -Xarch_host); device code is built as usual
    flags = ["--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-ffp-contract=off", "-Xclang", "-target-feature", "-Xclang",
             "-packed-fp32-ops", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
             "-fno-sanitize-recover=undefined", "-Wno-unused-function", "-Wno-pass-failed"]

    def compile_one(path):
        obj = str(tmp_path / (os.path.basename(path) + ".o"))
        res = _run(["hipcc", *flags, *inc, "-c", path, "-o", obj])
        assert res.returncode == 0, res.stderr[-4000:]
        return obj

    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
        objs = list(pool.map(compile_one, src))
    drv = str(tmp_path / "host_driver.o")
    res = _run(["hipcc", "-O1", "-g", "-std=c++17", "-fno-gpu-sanitize", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                *inc, "-x", "c++", "-c", os.path.join(SAN, "host_driver.cpp"), "-o", drv])
    assert res.returncode == 0, res.stderr[-4000:]
    exe = str(tmp_path / "host_san")
    res = _run(["hipcc", "--offload-arch=gfx950", "-fno-gpu-sanitize", "-fsanitize=address,undefined", *objs, drv, "-o", exe])
    assert res.returncode == 0, res.stderr[-4000:]
    run = _run([exe], env=dict(os.environ, ASAN_OPTIONS="detect_leaks=0"))
    assert run.returncode == 0 and "host sanitizer run ok" in run.stdout, run.stdout[-3000:] + run.stderr[-4000:]
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr
