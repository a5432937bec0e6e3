"""Compile the CPU oracle (plain C, gcc) into oracle/libhb_ref.so.

Test infrastructure: the product library is built elsewhere and never links this.
Run as `python -m oracle.build` or call `build()`.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCES = [os.path.join(HERE, "hb_ref.c"), os.path.join(HERE, "hb_ref_mp.c")]
LIBRARY = os.path.join(HERE, "libhb_ref.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIBRARY) and all(os.path.getmtime(LIBRARY) >= os.path.getmtime(f) for f in SOURCES):
        return LIBRARY
    tmp = LIBRARY + ".tmp.%d" % os.getpid()
    cmd = ["gcc", "-std=c11", "-O2", "-Wall", "-Wextra", "-fPIC", "-shared"] + SOURCES + ["-o", tmp, "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(tmp, LIBRARY)
    return LIBRARY


if __name__ == "__main__":
    print(build())
