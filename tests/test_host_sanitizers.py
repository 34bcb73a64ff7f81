"""The CPU oracle and the library's host-side scheduler under AddressSanitizer and UBSan.

Builds tests/sanitize/host_driver.cpp together with oracle/*.c and csrc/lwp_plan.cpp (host code only,
no HIP) with -fsanitize=address,undefined and runs it: any out-of-bounds access, leak of a freed
table, or signed overflow inside the oracle ends the run with a report."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


def test_oracle_and_scheduler_under_asan_ubsan(tmp_path):
    objs = []
    for src in ("oracle/lwp_oracle.c", "oracle/cost_model_oracle.c"):
        obj = tmp_path / (os.path.basename(src) + ".o")
        subprocess.run(["gcc", "-std=c11", "-fopenmp", "-Wall", "-Wextra", *SAN, "-c", os.path.join(ROOT, src), "-o", str(obj)],
                       check=True)
        objs.append(str(obj))
    inc = ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_1802_04924_amd", "csrc")]
    exe = tmp_path / "host_driver"
    subprocess.run(["g++", "-std=c++17", "-fopenmp", "-Wall", *SAN, *inc,
                    os.path.join(ROOT, "tests", "sanitize", "host_driver.cpp"),
                    os.path.join(ROOT, "paper_1802_04924_amd", "csrc", "lwp_plan.cpp"), *objs, "-o", str(exe)], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="2")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "sanitized host run ok" in r.stdout
