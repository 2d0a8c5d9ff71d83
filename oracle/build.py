"""Compile the C oracle into oracle/libkvs_oracle.so with gcc (test infrastructure)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "kvs_oracle.c")
LIB = os.path.join(HERE, "libkvs_oracle.so")


def build(force: bool = True) -> str:
    if os.environ.get("KVS_ORACLE_LIBRARY"):          # another build of the same source (the sanitizer run)
        return os.environ["KVS_ORACLE_LIBRARY"]
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
