"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer: oracle/taco_ref.cpp is compiled, with both,
into a driver that runs every entry point over every block size, mode, code book and a set of ragged lengths
(tests/oracle_sanitize/driver.cpp).  Any out-of-bounds access, overflow or other undefined behaviour aborts it."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    # the sanitizer runtime is linked statically so that it does not depend on its place in the list of preloaded libraries
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           "-fopenmp", "-ffp-contract=off", os.path.join(ROOT, "oracle", "taco_ref.cpp"),
           os.path.join(ROOT, "tests", "oracle_sanitize", "driver.cpp"), "-o", exe]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0")
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert res.returncode == 0, res.stdout[-2000:]
    assert "oracle_sanitize: ok" in res.stdout
