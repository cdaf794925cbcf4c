"""The C ABI's host code (argument checks, plan cache, scratch limits, allocation-failure paths) built for
the host alone, against stand-ins for the HIP runtime and the kernel launchers, under the address and
undefined-behaviour sanitizers; the driver is plain C, so the header is checked as C99 on the way."""
import os
import shutil
import subprocess
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "host_abi")


@pytest.mark.skipif(shutil.which("g++") is None or shutil.which("gcc") is None, reason="needs gcc and g++")
def test_host_side_of_the_abi_under_sanitizers(tmp_path):
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
    csrc = os.path.join(ROOT, "paper_2604_14156_amd", "csrc")
    inc = ["-I", HERE, "-I", csrc, "-I", os.path.join(ROOT, "include")]
    objs = []
    for src, cc, lang in ((os.path.join(csrc, "cs_api.hip"), "g++", ["-x", "c++", "-std=c++17"]),
                          (os.path.join(HERE, "standin_launchers.cpp"), "g++", ["-std=c++17"]),
                          (os.path.join(HERE, "driver.c"), "gcc", ["-std=c99", "-D_ISOC11_SOURCE", "-Wall", "-Werror"])):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        r = subprocess.run([cc] + lang + san + inc + ["-c", src, "-o", obj], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-3000:]
        objs.append(obj)
    exe = str(tmp_path / "host_abi")
    r = subprocess.run(["g++"] + san + objs + ["-o", exe], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)                     # the sanitizer runtime has to come first in the process
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, (r.stdout + r.stderr)[-4000:]
    assert "host ABI checks passed" in r.stdout
