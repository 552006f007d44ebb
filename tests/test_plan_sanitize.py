"""The host-side planning code (csrc/hyd_plan.cpp) under AddressSanitizer and
UndefinedBehaviorSanitizer, driven from plain C through include/hyd_plan.h (which also checks that
both headers are valid C): any report ends the run with a non-zero status."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def test_planner_is_clean_under_asan_and_ubsan(tmp_path):
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-g", "-O1"]
    obj_c, obj_cpp, exe = (str(tmp_path / n) for n in ("driver.o", "plan.o", "plan_sanitize"))
    inc = ["-I", os.path.join(ROOT, "include")]
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", *san, *inc, "-c", os.path.join(HERE, "plan_sanitize_driver.c"), "-o", obj_c])
    subprocess.check_call(["g++", "-std=c++17", "-Wall", *san, *inc, "-c",
                           os.path.join(ROOT, "paper_2412_07894_amd", "csrc", "hyd_plan.cpp"), "-o", obj_cpp])
    subprocess.check_call(["g++", *san, "-static-libasan", obj_c, obj_cpp, "-o", exe])
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert r.returncode == 0, r.stdout
    assert "status 0" in r.stdout and "ERROR" not in r.stdout, r.stdout
