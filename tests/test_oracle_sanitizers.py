"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): the C
driver tests/oracle_sanitize.c is compiled together with oracle/adamas_oracle.c and run as a plain
program, so no sanitizer runtime has to be loaded into Python."""

import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    cmd = ["gcc", "-std=c99", "-O1", "-g", "-fno-omit-frame-pointer", "-fopenmp",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-Wall", "-Wextra",
           os.path.join(ROOT, "tests", "oracle_sanitize.c"),
           os.path.join(ROOT, "oracle", "adamas_oracle.c"), "-o", exe, "-lm"]
    subprocess.run(cmd, check=True)
    # (the environment may preload a library of its own into every process: the sanitizer runtime
    # then is not the first in the link order, which is all right here)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               OMP_NUM_THREADS="2")
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env,
                       timeout=300)
    assert r.returncode == 0 and "oracle_sanitize: ok" in r.stdout, r.stdout[-4000:]
