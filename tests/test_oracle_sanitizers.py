"""The oracle's C code under AddressSanitizer and UndefinedBehaviorSanitizer: the library is built
again with -fsanitize=address,undefined and every pin test of the oracle runs against that build in
a child process (the sanitizer runtime has to be loaded before the interpreter's own libraries)."""
import glob
import os
import subprocess
import sys

from oracle import build as oracle_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_pins_pass_under_asan_and_ubsan(tmp_path):
    lib = oracle_build.build_sanitized(str(tmp_path / "libratsparse_ref_san.so"))
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True, check=True).stdout.strip()
    assert os.path.isabs(asan) and os.path.exists(asan), asan
    env = dict(os.environ)
    env["RATSPARSE_REF_LIB"] = lib
    env["LD_PRELOAD"] = asan + ((":" + env["LD_PRELOAD"]) if env.get("LD_PRELOAD") else "")
    # the interpreter and the numeric libraries are not instrumented: no leak report, but any bad access or
    # undefined operation inside the oracle stops the child at once
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    me = os.path.abspath(__file__)
    files = sorted(f for f in glob.glob(os.path.join(ROOT, "tests", "test_oracle_*.py")) if os.path.abspath(f) != me)
    assert len(files) >= 5
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu"] + files,
                       env=env, cwd=ROOT, capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "AddressSanitizer" not in tail and "runtime error" not in tail, tail
