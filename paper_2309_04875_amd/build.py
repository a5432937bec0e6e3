"""Build paper_2309_04875_amd/libhb.so (the library) and libhb_probes.so (bench.py's measurement aids, a separate
library that the product does not load) from csrc/ with hipcc for gfx950 (cross-compiles without a GPU).

The group kernels exist once per (mode, slice width); hb_launch_part.hip is compiled once per mode and
width range so that the parts build in parallel.  Objects go to a temporary directory; only the
library is left in the tree.  Run as `python -m paper_2309_04875_amd.build`.
"""
import os
import shutil
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIBRARY = os.path.join(HERE, "libhb.so")
PROBES_LIBRARY = os.path.join(HERE, "libhb_probes.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    "-fvisibility=hidden",
    "-Wall",
    # packed FP32 instructions are not to be generated on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]

MODES = (0, 1, 2, 3, 4)                                 # DReLU, ReLU, sign shares; DReLU, ReLU on the shared-mask layout
WIDTH_RANGES = ((1, 16), (17, 32), (33, 48), (49, 64))
MP_PARTIES = (3, 4)                                     # multi-party kernels (two parties: the kernels above)
MP_WIDTH_RANGES = ((1, 8), (9, 16), (17, 32), (33, 48), (49, 64))


def _hipcc():
    return os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _compile(args):
    src, obj, defines = args
    cmd = [_hipcc()] + HIPCC_FLAGS + ["-D%s=%s" % kv for kv in defines] + ["-c", src, "-o", obj]
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines() if "not a recognized feature for this target" not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build(verbose: bool = False, jobs: int = 0) -> str:
    jobs = jobs or min(8, os.cpu_count() or 1)
    work = tempfile.mkdtemp(prefix="hb_build_")
    try:
        probes = (os.path.join(CSRC, "hb_probes.hip"), os.path.join(work, "hb_probes.o"), [])
        units = [(os.path.join(CSRC, "hb_api.hip"), os.path.join(work, "hb_api.o"), [])]
        for mode in MODES:
            for lo, hi in WIDTH_RANGES:
                units.append((os.path.join(CSRC, "hb_launch_part.hip"),
                              os.path.join(work, "part_m%d_w%d.o" % (mode, lo)),
                              [("HB_PART_MODE", mode), ("HB_PART_LO", lo), ("HB_PART_HI", hi)]))
        for parties in MP_PARTIES:
            for lo, hi in MP_WIDTH_RANGES:
                units.append((os.path.join(CSRC, "hb_mp_part.hip"),
                              os.path.join(work, "mp_p%d_w%d.o" % (parties, lo)),
                              [("HB_PART_PARTIES", parties), ("HB_PART_LO", lo), ("HB_PART_HI", hi)]))
        with ThreadPoolExecutor(max_workers=jobs) as pool:
            for out in pool.map(_compile, [probes] + units):
                if verbose and out.strip():
                    print(out)
        for objects, library in (([u[1] for u in units], LIBRARY), ([probes[1]], PROBES_LIBRARY)):
            tmp = library + ".tmp.%d" % os.getpid()
            cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC"] + objects + ["-o", tmp]
            subprocess.run(cmd, check=True)
            os.replace(tmp, library)
    finally:
        shutil.rmtree(work, ignore_errors=True)
    return LIBRARY


if __name__ == "__main__":
    print(build(verbose=True))
