"""Address and undefined-behaviour sanitizers on the host-side planner (no GPU code is compiled or run)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_1711_01348_amd", "csrc")


def test_planner_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "plan_sanitize")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-static-libasan", "-static-libubsan",
           os.path.join(CSRC, "plan.cpp"), os.path.join(CSRC, "derived.cpp"), os.path.join(CSRC, "families.cpp"),
           os.path.join(ROOT, "tests", "host_sanitize_driver.cpp"), "-o", exe]
    subprocess.run(cmd, check=True)
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0"
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    sys.stdout.write(r.stdout)
    sys.stderr.write(r.stderr[-4000:])
    assert r.returncode == 0, r.returncode
    assert "sanitizer driver ok" in r.stdout
