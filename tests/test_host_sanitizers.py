"""AddressSanitizer + UndefinedBehaviorSanitizer build of the host code (CPU only).

tests/sanitize/host_checks.cpp drives the C oracle and the library's host translation units (layout builder, cache
geometry, and the argument checks of the entry points with the HIP runtime stubbed out) over a spread of shapes, and
cross-checks mask and tile schedule against the oracle's predicate.  Built and run here as one executable:

    gcc -c -O1 -g -fsanitize=address,undefined -fno-sanitize-recover=all -fopenmp oracle/ksa_oracle.c
    g++ -O1 -g -std=c++17 -fsanitize=address,undefined -fno-sanitize-recover=all -fopenmp \\
        -I tests/sanitize/hip_stub -I include -I paper_2604_24432_amd/csrc \\
        tests/sanitize/host_checks.cpp paper_2604_24432_amd/csrc/ksa_layout.cpp paper_2604_24432_amd/csrc/ksa_api.cpp \\
        ksa_oracle.o -o host_checks && ./host_checks

Any sanitizer finding aborts the program with a non-zero status.
"""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fopenmp"]


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    obj = str(tmp_path / "ksa_oracle.o")
    exe = str(tmp_path / "host_checks")
    subprocess.run(["gcc", "-c", "-std=c11", *SAN, os.path.join(ROOT, "oracle", "ksa_oracle.c"), "-o", obj], check=True)
    csrc = os.path.join(ROOT, "paper_2604_24432_amd", "csrc")
    subprocess.run(["g++", "-std=c++17", *SAN, "-I", os.path.join(ROOT, "tests", "sanitize", "hip_stub"),
                    "-I", os.path.join(ROOT, "include"), "-I", csrc,
                    os.path.join(ROOT, "tests", "sanitize", "host_checks.cpp"), os.path.join(csrc, "ksa_layout.cpp"),
                    os.path.join(csrc, "ksa_api.cpp"), obj, "-o", exe, "-lm"], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert res.returncode == 0, res.stdout[-3000:] + res.stderr[-3000:]
    assert "host checks passed" in res.stdout
