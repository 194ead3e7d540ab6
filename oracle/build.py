"""Compile the CPU oracle (plain C, gcc) into oracle/libta_oracle.so.

Test infrastructure only; see the header of ta_oracle.c.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "ta_oracle.c")
LIB = os.path.join(HERE, "libta_oracle.so")


SAN_LIB = os.path.join(HERE, "libta_oracle_san.so")


def build(verbose: bool = False, sanitize: bool = False) -> str:
    """sanitize=True: the same source with AddressSanitizer and UBSan (host only), for the test that
    runs the pins against it; a process that loads it must have the ASan runtime preloaded."""
    if sanitize:
        cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-fsanitize=address,undefined",
               "-fno-sanitize-recover=all", "-Wall", "-Wextra", SRC, "-o", SAN_LIB, "-lm"]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        return SAN_LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC",
           "-Wall", "-Wextra", SRC, "-o", LIB, "-lm"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
