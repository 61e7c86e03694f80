"""The host side of the library (argument checks, workspace layout, span plan, the schedule of both passes) under
AddressSanitizer and UBSan.  Built without device code: the kernel launchers are replaced by no-op stubs
(tests/sanitize/stub_launchers.cpp), so the whole forward+backward schedule runs on the CPU with never-dereferenced
"device" pointers, over shapes up to the size limits (960 sentences, 1024 words, the headline grammar)."""
import os
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2310_14997_amd", "csrc")
SAN = os.path.join(ROOT, "tests", "sanitize")


def test_host_scheduler_is_clean_under_asan_and_ubsan():
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "host_checks")
        cmd = [hipcc, "--cuda-host-only", "-O1", "-g", "-std=c++17", "-w", "-DSPCFG_HOST_CHECKS_BUILD",
               "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
               "-I", CSRC]
        for src in (os.path.join(CSRC, "spcfg_api.hip"), os.path.join(SAN, "stub_launchers.cpp"),
                    os.path.join(SAN, "host_checks.cpp")):
            cmd += ["-x", "hip", src]
        cmd += ["-o", exe]
        subprocess.check_call(cmd, cwd=tmp)
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1")
        env.pop("LD_PRELOAD", None)  # the sanitizer runtime has to come first in the library list
        res = subprocess.run([exe], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
        assert res.returncode == 0, res.stdout[-4000:]
        assert "host checks passed" in res.stdout, res.stdout[-2000:]
