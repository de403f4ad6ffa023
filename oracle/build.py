"""Compile the C oracle with gcc into oracle/liborbit_oracle.so (test infrastructure)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "orbit_oracle.c")
LIB = os.path.join(HERE, "liborbit_oracle.so")


def build(force: bool = False) -> str:
    """Path of the built oracle library.  ORBIT_ORACLE_LIB names a library to use instead: the
    mutation test points it at deliberately broken builds to show that the pins reject them."""
    override = os.environ.get("ORBIT_ORACLE_LIB")
    if override:
        return override
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
           "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
