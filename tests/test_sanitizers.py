"""The oracle and the host logic of the library under AddressSanitizer + UndefinedBehaviorSanitizer.

tests/native/policy_sanitize.cpp links oracle/cascade_oracle.c with csrc/structure.cpp and
csrc/simulate.cpp (the score-independent structure of the update and the host replay of its
score-dependent part, which runs the routines of plan_core.h that the device kernels run) and
compares the two over seeded random geometries.  Host code only: no device is touched."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANG = "/opt/rocm/lib/llvm/bin/clang"


@pytest.mark.skipif(not os.path.exists(CLANG), reason="the ROCm clang is not installed")
def test_policy_under_address_and_ub_sanitizers(tmp_path):
    csrc = os.path.join(ROOT, "paper_2406_17808_amd", "csrc")
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
    objs = []
    for src, lang in ((os.path.join(ROOT, "oracle", "cascade_oracle.c"), ["-x", "c", "-std=c11"]),
                      (os.path.join(csrc, "structure.cpp"), ["-x", "c++", "-std=c++17"]),
                      (os.path.join(csrc, "simulate.cpp"), ["-x", "c++", "-std=c++17"]),
                      (os.path.join(ROOT, "tests", "native", "policy_sanitize.cpp"), ["-x", "c++", "-std=c++17"])):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        # the HIP headers are only needed for their host-side declarations (no device code in these files)
        subprocess.check_call([CLANG] + lang + san + ["-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-Wall",
                                                      "-Wno-unknown-pragmas", "-c", src, "-o", obj])
        objs.append(obj)
    exe = str(tmp_path / "policy_sanitize")
    subprocess.check_call([CLANG + "++"] + san + objs + ["-o", exe, "-lm"])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:verify_asan_link_order=0:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    env.pop("LD_PRELOAD", None)
    res = subprocess.run([exe, "40"], env=env, capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "41 cases, 0 failed" in res.stdout
    shutil.rmtree(tmp_path, ignore_errors=True)
