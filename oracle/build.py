"""Compiles the C oracle into oracle/libftp_oracle.so (gcc, OpenMP)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libftp_oracle.so")


def build(force=True):
    src = os.path.join(HERE, "ftp_oracle.c")
    inc = os.path.join(HERE, "ftp_oracle_impl.inc")
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(os.path.getmtime(src), os.path.getmtime(inc)):
        return LIB
    cmd = ["gcc", "-O3", "-fopenmp", "-shared", "-fPIC", "-fno-fast-math", "-ffp-contract=off",
           src, "-o", LIB]
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build())
