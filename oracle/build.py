"""Build the CPU oracle (test infrastructure) into oracle/libratsparse_ref.so with gcc."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCES = ["ref_util.c", "ref_scan.c", "ref_quest.c", "ref_attn.c", "ref_moba.c", "ref_snapkv.c"]
LIB = os.path.join(HERE, "libratsparse_ref.so")


def build(force: bool = True) -> str:
    srcs = [os.path.join(HERE, s) for s in SOURCES]
    deps = srcs + [os.path.join(HERE, "ratsparse_ref.h")]
    if not force and os.path.exists(LIB) and all(
        os.path.getmtime(LIB) >= os.path.getmtime(d) for d in deps
    ):
        return LIB
    # -ffp-contract=off: keep every product and sum a separately rounded double
    # operation, as written.
    cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
           "-Wall", "-Wextra", "-o", LIB] + srcs + ["-lm"]
    subprocess.run(cmd, check=True)
    return LIB


def build_sanitized(out: str) -> str:
    """The same sources with AddressSanitizer and UndefinedBehaviorSanitizer (host code only), into
    `out`; a test loads it in a child process through RATSPARSE_REF_LIB."""
    srcs = [os.path.join(HERE, s) for s in SOURCES]
    cmd = ["gcc", "-std=c11", "-O1", "-g", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
           "-Wall", "-Wextra", "-o", out] + srcs + ["-lm"]
    subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    print(build(force="--if-stale" not in sys.argv))
