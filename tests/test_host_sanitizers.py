"""The library's host code (argument validation, size queries, plan arithmetic, weight computation) under
AddressSanitizer and UndefinedBehaviorSanitizer.

Every HIP source is compiled once more with the sanitizers switched on for the HOST pass only (the device
code is compiled as usual but never run) and linked with tests/host_sanitize/abi_host_checks.cpp into an
executable, so the sanitizer runtime is linked in rather than preloaded.  The driver calls only paths that
return before any GPU call, so this needs no GPU.  The sanitizers end the process on a finding.
"""
import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

from paper_2601_07396_amd import build as pkg_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANGXX = "/opt/rocm/llvm/bin/clang++"
HOST_SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
            "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-g"]


def _run(cmd):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    assert res.returncode == 0, " ".join(cmd) + "\n" + out[-4000:]
    return out


@pytest.mark.timeout(900)
def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    if not os.path.exists(CLANGXX):
        pytest.skip("ROCm clang++ not found")
    srcs = sorted(glob.glob(os.path.join(ROOT, "paper_2601_07396_amd", "csrc", "*.hip")))
    assert srcs
    # same flags as the product build, except -O1: only the host half of these objects ever runs
    flags = [f for f in pkg_build.HIPCC_FLAGS if f != "-O3"] + ["-O1"] + HOST_SAN
    objs = [str(tmp_path / (os.path.basename(s)[:-4] + ".o")) for s in srcs]
    with ThreadPoolExecutor(max_workers=min(len(srcs), os.cpu_count() or 1, 8)) as pool:
        list(pool.map(lambda so: _run(["hipcc", *flags, "-c", "-o", so[1], so[0]]), zip(srcs, objs)))
    drv = str(tmp_path / "abi_host_checks.o")
    _run([CLANGXX, "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
          "-I", os.path.join(ROOT, "include"), "-c", "-o", drv,
          os.path.join(ROOT, "tests", "host_sanitize", "abi_host_checks.cpp")])
    exe = str(tmp_path / "abi_host_checks")
    _run([CLANGXX, "-fsanitize=address,undefined", "-o", exe, drv, *objs,
          "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib"])
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert res.returncode == 0, res.stdout[-4000:]
    assert "host ABI checks passed" in res.stdout
    assert "runtime error" not in res.stdout and "AddressSanitizer" not in res.stdout
