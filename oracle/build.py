"""Compile the CPU oracle (plain C, gcc) into oracle/libhb_ref.so.

Test infrastructure: the product library is built elsewhere and never links this.
Run as `python -m oracle.build` or call `build()`.

With HB_ORACLE_SANITIZE=1 in the environment (or `build(sanitize=True)`) a second library,
oracle/libhb_ref_san.so, is built with AddressSanitizer and UndefinedBehaviorSanitizer
(`-fsanitize=address,undefined -fno-sanitize-recover=all`: any report aborts the process) and
`oracle.lib()` loads that one; the process must then start with the sanitizer runtime preloaded
(`LD_PRELOAD=$(gcc -print-file-name=libasan.so)`), which tests/test_oracle_sanitized.py does for a
child process.  CPU only.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCES = [os.path.join(HERE, "hb_ref.c"), os.path.join(HERE, "hb_ref_mp.c")]
LIBRARY = os.path.join(HERE, "libhb_ref.so")
SANITIZED_LIBRARY = os.path.join(HERE, "libhb_ref_san.so")
SANITIZE_FLAGS = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g"]


def sanitize_requested() -> bool:
    return os.environ.get("HB_ORACLE_SANITIZE", "0") not in ("", "0")


def sanitizer_runtime() -> str:
    """Path of the AddressSanitizer runtime that a process loading the sanitized oracle must preload."""
    return subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, stdout=subprocess.PIPE,
                          text=True).stdout.strip()


def build(force: bool = True, sanitize: bool = None) -> str:
    if sanitize is None:
        sanitize = sanitize_requested()
    library = SANITIZED_LIBRARY if sanitize else LIBRARY
    if not force and os.path.exists(library) and all(os.path.getmtime(library) >= os.path.getmtime(f) for f in SOURCES):
        return library
    tmp = library + ".tmp.%d" % os.getpid()
    flags = ["-O1"] + SANITIZE_FLAGS if sanitize else ["-O2"]
    cmd = ["gcc", "-std=c11", "-Wall", "-Wextra", "-fPIC", "-shared"] + flags + SOURCES + ["-o", tmp, "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(tmp, library)
    return library


if __name__ == "__main__":
    print(build())
