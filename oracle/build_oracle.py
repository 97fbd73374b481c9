"""Builds the CPU oracle (test infrastructure) into two shared libraries:
liborc_f64.so (arithmetic in double, the parity reference) and liborc_f32.so
(the same source with float arithmetic)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
FLAGS = ["-O3", "-fopenmp", "-mavx2", "-mfma", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra", "-Wno-unused-parameter"]


def build(verbose=False):
    src = os.path.join(HERE, "gr4ad_oracle.c")
    for name, extra in (("liborc_f64.so", []), ("liborc_f32.so", ["-DORC_REAL_FLOAT"])):
        cmd = ["gcc", *FLAGS, *extra, src, "-o", os.path.join(HERE, name), "-lm"]
        if verbose:
            print(" ".join(cmd))
        subprocess.check_call(cmd)


if __name__ == "__main__":
    build(verbose=True)
