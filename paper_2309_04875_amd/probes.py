"""ctypes access to libhb_probes.so: bench.py's measurement aids (clock probe, vector-ALU issue-cost streams,
a 2-in / 2-out streaming kernel).  Not part of the library's interface; nothing in the product imports this."""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIBRARY = os.path.join(HERE, "libhb_probes.so")

_lib = None


def load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIBRARY):
        raise ImportError("%s is missing: build it with `python -m paper_2309_04875_amd.build`" % LIBRARY)
    lib = ctypes.CDLL(LIBRARY)
    vp, u64, ci = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int
    lib.hbp_issue_probe_count.restype = ci
    lib.hbp_issue_class_count.restype = ci
    lib.hbp_issue_probe_name.restype = ctypes.c_char_p
    lib.hbp_issue_probe_name.argtypes = [ci]
    lib.hbp_issue_load.restype = ci
    lib.hbp_issue_load.argtypes = [ci, ci, ci, ci, vp]
    lib.hbp_issue_probe.restype = ci
    lib.hbp_issue_probe.argtypes = [ci, ci, ci, ctypes.POINTER(ctypes.c_double)]
    lib.hbp_clock_probe.restype = ci
    lib.hbp_clock_probe.argtypes = [u64, vp, vp]
    lib.hbp_stream_copy.restype = ci
    lib.hbp_stream_copy.argtypes = [ci, ci, vp, vp, vp, vp, u64, vp]
    _lib = lib
    return lib


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def issue_probe_names():
    lib = load()
    return [lib.hbp_issue_probe_name(i).decode() for i in range(lib.hbp_issue_probe_count())]


def issue_class_count():
    return int(load().hbp_issue_class_count())


def issue_probe(index, waves_per_simd=8, iters=4096):
    """{ms, mhz, cycles_per_instruction, instructions_per_wave} of one timed launch of probe `index`."""
    res = (ctypes.c_double * 4)()
    st = load().hbp_issue_probe(int(index), int(waves_per_simd), int(iters), res)
    if st != 0:
        raise RuntimeError("hbp_issue_probe(%d) failed: %d" % (index, st))
    return {"ms": res[0], "mhz": res[1], "cycles_per_instruction": res[2], "instructions_per_wave": res[3]}


def issue_load(index, waves_per_simd, iters, launches):
    st = load().hbp_issue_load(int(index), int(waves_per_simd), int(iters), int(launches), _stream())
    if st != 0:
        raise RuntimeError("hbp_issue_load(%d) failed: %d" % (index, st))


def clock_probe(spins, stamps):
    """Enqueue the one-wavefront clock probe on torch's current stream; stamps: 2-entry int64 CUDA tensor."""
    st = load().hbp_clock_probe(int(spins), stamps.data_ptr(), _stream())
    if st != 0:
        raise RuntimeError("hbp_clock_probe failed: %d" % st)
    return stamps


def stream_copy(x0, x1, o0, o1, nontemporal=True, xcd_contiguous=False):
    st = load().hbp_stream_copy(int(nontemporal), int(xcd_contiguous), x0.data_ptr(), x1.data_ptr(), o0.data_ptr(),
                                o1.data_ptr(), x0.numel(), _stream())
    if st != 0:
        raise RuntimeError("hbp_stream_copy failed: %d" % st)
