"""The library's host code under AddressSanitizer and UndefinedBehaviorSanitizer: every translation
unit is compiled once more with the host pass instrumented (the gfx950 pass untouched), linked
into a driver (tests/host/sanitize_driver.cpp) that walks descriptor validation, buffer sizing,
launch geometry and every argument check that returns before a launch.  Needs no GPU."""
import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

from paper_2508_04257_amd import build as kbuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-gpu-sanitize", "-fno-sanitize-recover=undefined", "-g", "-O1"]


def test_host_paths_are_clean_under_asan_and_ubsan(tmp_path):
    if shutil.which("hipcc") is None:
        pytest.skip("no hipcc")
    common = [f for f in kbuild.COMMON if f != "-O3"]

    def compile_one(name):
        obj = str(tmp_path / name.replace(".hip", ".o"))
        cmd = ["hipcc", *common, *kbuild.SOURCES[name], *SAN, "-c", os.path.join(kbuild.CSRC, name), "-o", obj]
        res = subprocess.run(cmd, capture_output=True, text=True)
        assert res.returncode == 0, res.stderr[-3000:]
        return obj

    with ThreadPoolExecutor(max_workers=8) as pool:
        objs = list(pool.map(compile_one, kbuild.SOURCES))
    drv = str(tmp_path / "driver.o")
    res = subprocess.run(["hipcc", "-x", "c++", "-std=c++17", *SAN, "-I", os.path.join(ROOT, "include"), "-c",
                          os.path.join(ROOT, "tests", "host", "sanitize_driver.cpp"), "-o", drv], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-3000:]
    exe = str(tmp_path / "sanitize_driver")
    res = subprocess.run(["hipcc", "--offload-arch=gfx950", *SAN, *objs, drv, "-o", exe], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-4000:])
    assert "host checks passed" in run.stdout
