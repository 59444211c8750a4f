"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only).

tests/sanitize/driver.c includes the oracle's C source and links the library's
host-only schedule (csrc/skd_schedule.cpp); it walks the schedule pins (also at
the int32 extremes) and the cached == brute-force decoder pin on a tiny model.
Built with -fsanitize=address,undefined -fno-sanitize-recover=all, any
out-of-bounds access, signed overflow, leak or use after free ends it with a
non-zero status.
"""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]


def test_oracle_and_schedule_under_asan_ubsan(tmp_path):
    drv_o, sch_o, exe = (str(tmp_path / n) for n in ("driver.o", "schedule.o", "driver"))
    subprocess.run(["gcc", "-std=gnu99", "-Wall", *SAN, "-fopenmp", "-c",
                    os.path.join(ROOT, "tests", "sanitize", "driver.c"), "-o", drv_o], check=True)
    subprocess.run(["g++", "-std=c++17", "-Wall", *SAN, "-c",
                    os.path.join(ROOT, "paper_2307_02628_amd", "csrc", "skd_schedule.cpp"), "-o", sch_o], check=True)
    subprocess.run(["g++", *SAN, "-fopenmp", drv_o, sch_o, "-lm", "-o", exe], check=True)
    # a library preloaded into every process may precede the sanitizer runtime: do not insist on the link order
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="2")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "all checks passed" in res.stdout
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr
