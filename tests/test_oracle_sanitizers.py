"""CPU sanitizer tier: the checker built with AddressSanitizer and UndefinedBehaviorSanitizer
(gcc, CPU only) must pass every pin of the CPU suite without a report.  The sanitized library
is loaded by a child pytest process through OVF_LIB, with the sanitizer runtime put in front
of whatever is preloaded already."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(bool(os.environ.get("OVF_LIB")), reason="already inside the sanitizer run")
def test_checker_under_asan_and_ubsan(tmp_path):
    lib = str(tmp_path / "libvf_oracle_san.so")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-fno-fast-math", "-ffp-contract=off",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
           "-o", lib, os.path.join(ROOT, "oracle", "vf_oracle.c"), "-lm"]
    subprocess.run(cmd, check=True)
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True, check=True).stdout.strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("no AddressSanitizer runtime next to gcc")
    env = dict(os.environ)
    env["OVF_LIB"] = lib
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=99"   # (the interpreter's own leaks are not ours)
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests"), "-x", "-q", "-m", "not gpu",
                        "-k", "oracle and not sanitizers", "-p", "no:cacheprovider"],
                       capture_output=True, text=True, env=env, cwd=ROOT, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "AddressSanitizer" not in tail and "runtime error" not in tail, tail
