"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only): the oracle and the library's host side
(HARVEST_FLAG_NO_DEVICE: no HIP call is made) are rebuilt with the sanitizers and driven in lock step by
tests/sanitize/driver.c.  Device code is not sanitized: only the host pass of hipcc gets the flags."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g"]


@pytest.mark.skipif(shutil.which("hipcc") is None or shutil.which("gcc") is None, reason="needs hipcc and gcc")
def test_host_logic_and_oracle_under_sanitizers(tmp_path):
    lib = tmp_path / "libharvest_san.so"
    # -DHARVEST_FAULT_INJECTION: this build (and only this one) can be told to fail at its n-th device step, which is how
    # the driver reaches the roll-back code of place / evict / revoke
    hip = ["hipcc", "--offload-arch=gfx950", "-O1", "-std=c++17", "-fPIC", "-shared", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-DHARVEST_FAULT_INJECTION"]
    for f in SAN:
        hip += ["-Xarch_host", f]
    hip += ["-o", str(lib), os.path.join(ROOT, "paper_2602_00328_amd", "csrc", "harvest.hip")]
    subprocess.check_call(hip)
    orc = tmp_path / "liboracle_san.so"
    # the same compiler family for everything: one sanitizer runtime serves the whole process (OpenMP pragmas are left
    # out of this build: the loops they mark run serially)
    subprocess.check_call(["hipcc", "-x", "c", "-fno-gpu-sanitize", "-O1", "-std=c99", "-Wno-unknown-pragmas", "-shared", "-fPIC", *SAN, "-o", str(orc),
                           os.path.join(ROOT, "oracle", "harvest_oracle.c")])
    exe = tmp_path / "driver"
    subprocess.check_call(["hipcc", "-x", "c", "-fno-gpu-sanitize", "-O1", "-g", *SAN, "-I", os.path.join(ROOT, "include"),
                           os.path.join(ROOT, "tests", "sanitize", "driver.c"), "-x", "none", "-o", str(exe), str(lib), str(orc),
                           f"-Wl,-rpath,{tmp_path}"])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([str(exe)], env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-6000:]
    assert "sanitizer run: ok" in r.stdout and "injected faults rolled back" in r.stdout
