"""Builds liblstm_int_oracle.so (plain C, gcc -O2, OpenMP over batch rows).

TEST INFRASTRUCTURE.  Run: python oracle/build.py
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "liblstm_int_oracle.so")
SAN_LIB = os.path.join(HERE, "liblstm_int_oracle_san.so")


def _sources():
    """The LSTM oracle, and the GRU and the SRU assembled from the same primitives."""
    return [os.path.join(HERE, n) for n in ("lstm_int_oracle.c", "gru_int_oracle.c", "sru_int_oracle.c")]


def build_sanitized():
    """The same source under AddressSanitizer and UndefinedBehaviorSanitizer, errors
    fatal: the oracle's claims of 64-bit headroom (Sec. 3.1.1 overflow model) and
    its indexing are then checked by the machine.  Loaded by a process that has
    the sanitizer runtime preloaded (tests/test_sanitizers.py)."""
    cmd = ["gcc", "-std=c11", "-O1", "-g", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-Wall", "-Wextra", "-o", SAN_LIB] + _sources() + ["-lm"]
    subprocess.run(cmd, check=True)
    return SAN_LIB


def build(force=True):
    deps = _sources() + [os.path.join(HERE, n) for n in ("lstm_int_oracle.h", "gru_int_oracle.h", "sru_int_oracle.h")]
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(os.path.getmtime(d) for d in deps):
        return LIB
    cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
           "-Wall", "-Wextra", "-o", LIB] + _sources() + ["-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
