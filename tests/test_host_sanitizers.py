"""Host sanitizer build: the library's host units (1-SA, VBR build and packing, unpacking, blocking
curve, bounds audit, launch plan) and the C oracle compiled with -fsanitize=address,undefined into
one executable (tests/host_check.cpp) that compares the two bit for bit over seeded matrices.
No HIP unit is part of it and no GPU is touched; a sanitizer report or a mismatch fails the run."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2202_05868_amd", "csrc")


def test_host_units_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "host_check")
    obj = str(tmp_path / "oracle.o")
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
    subprocess.check_call(["gcc", "-std=c99", "-ffp-contract=off", "-c", os.path.join(ROOT, "oracle", "vbr_oracle.c"), "-o", obj] + san)
    subprocess.check_call(["g++", "-std=c++17", "-mpopcnt", "-pthread", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                           os.path.join(ROOT, "tests", "host_check.cpp"), os.path.join(CSRC, "sa1_reorder.cpp"),
                           os.path.join(CSRC, "vbr_build.cpp"), obj, "-o", exe, "-lm"] + san)
    env = {k: v for k, v in os.environ.items() if k != "VBR_SA1_THREADS"}
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1"
    res = subprocess.run([exe], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    sys.stdout.write(res.stdout[-4000:])
    assert res.returncode == 0, res.stdout[-4000:]
    assert "host_check ok" in res.stdout
