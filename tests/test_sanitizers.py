"""The CPU sanitizer leg: the oracle and the library's host-side arithmetic and
offline phase, rebuilt under AddressSanitizer + UndefinedBehaviorSanitizer with
errors fatal, run through the 9 variants, layer norm at N = 4096 on extreme rows
and accumulation depth 2^15 at the weight and input bounds (the overflow model of
Sec. 3.1.1: every intermediate the method names must fit the width the code
gives it -- a signed overflow or an oversized shift traps here)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))


def test_oracle_and_host_math_under_asan_ubsan():
    from oracle import build as obuild
    from paper_2101_05453_amd import build as lbuild

    orc_lib = obuild.build_sanitized()
    hm_lib = lbuild.build_hostmath(sanitize=True)
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True, check=True).stdout.strip()
    assert os.path.isabs(asan) and os.path.exists(asan), asan
    env = dict(os.environ)
    env["LSTM_INT_ORACLE_LIB"] = orc_lib
    # the sanitizer runtime has to be in the process before the sanitized libraries are loaded
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["OMP_NUM_THREADS"] = "4"
    r = subprocess.run([sys.executable, os.path.join(HERE, "san_driver.py"), hm_lib], env=env, capture_output=True,
                       text=True, timeout=900)
    assert r.returncode == 0 and "SAN DRIVER OK" in r.stdout, (r.returncode, r.stdout[-2000:], r.stderr[-4000:])
