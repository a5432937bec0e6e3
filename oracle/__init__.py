"""CPU oracle for reduced-ring secret-shared DReLU / ReLU (test infrastructure).

Thin ctypes/numpy access to oracle/hb_ref.c.  Only tests, the smoke check and the
benchmark's cpu_baseline leg import this package; the product library does not.
"""
import ctypes
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_lib = None

WHAT_DRELU, WHAT_RELU, WHAT_SUM, WHAT_SIGN, WHAT_SLICE = 0, 1, 2, 3, 4

_i64p = ctypes.POINTER(ctypes.c_int64)
_u64p = ctypes.POINTER(ctypes.c_uint64)
_u64 = ctypes.c_uint64
_int = ctypes.c_int


def lib():
    global _lib
    if _lib is None:
        from .build import build as _build_oracle
        path = _build_oracle(force=False)
        L = ctypes.CDLL(path)
        L.hb_ref_mix64.restype = _u64
        L.hb_ref_mix64.argtypes = [_u64]
        L.hb_ref_sm_next.restype = _u64
        L.hb_ref_sm_next.argtypes = [_u64p]
        L.hb_ref_sm.restype = _u64
        L.hb_ref_sm.argtypes = [_u64, _u64]
        L.hb_ref_tensor_seed.restype = _u64
        L.hb_ref_tensor_seed.argtypes = [_u64, _u64]
        L.hb_ref_opened_bits.restype = _u64
        L.hb_ref_opened_bits.argtypes = [_int, _int, _int, _u64]
        L.hb_ref_opened_bits_v.restype = _u64
        L.hb_ref_opened_bits_v.argtypes = [_int, _int, _int, _u64, _int]
        L.hb_ref_and_gate.restype = None
        L.hb_ref_and_gate.argtypes = [_u64] * 10 + [_u64p, _u64p]
        L.hb_ref_eval_range_v.restype = _int
        L.hb_ref_eval_range_v.argtypes = [_i64p, _i64p, _u64, _u64, _int, _int, _u64, _int, _int, _int, _i64p, _i64p]
        L.hb_ref_eval_at_v.restype = _int
        L.hb_ref_eval_at_v.argtypes = [_i64p, _i64p, _u64p, _u64, _int, _int, _u64, _int, _int, _int, _i64p, _i64p]
        L.hb_ref_drelu.restype = _int
        L.hb_ref_drelu.argtypes = [_i64p, _i64p, _u64, _int, _int, _u64, _int, _i64p, _i64p, _u64p]
        L.hb_ref_relu.restype = _int
        L.hb_ref_relu.argtypes = [_i64p, _i64p, _u64, _int, _int, _u64, _int, _i64p, _i64p, _u64p]
        L.hb_ref_eco_scan.restype = _int
        L.hb_ref_eco_scan.argtypes = [_i64p, _i64p, _u64, _u64, _int, _u64p]
        L.hb_ref_eco_choose.restype = _int
        L.hb_ref_eco_choose.argtypes = [_u64p, _int]
        L.hb_ref_wire_words.restype = _u64
        L.hb_ref_wire_words.argtypes = [_u64, _int, _int]
        L.hb_ref_relu_wire.restype = _int
        L.hb_ref_relu_wire.argtypes = [_i64p, _i64p, _u64, _int, _int, _u64, _u64p, _u64p]
        L.hb_ref_wire_words_v.restype = _u64
        L.hb_ref_wire_words_v.argtypes = [_u64, _int, _int, _int]
        L.hb_ref_relu_wire_v.restype = _int
        L.hb_ref_relu_wire_v.argtypes = [_i64p, _i64p, _u64, _int, _int, _u64, _int, _u64p, _u64p]
        _f32p = ctypes.POINTER(ctypes.c_float)
        L.hb_ref_share_f32.restype = _int
        L.hb_ref_share_f32.argtypes = [_f32p, _u64, _u64, _i64p, _i64p]
        L.hb_ref_reveal_f32.restype = _int
        L.hb_ref_reveal_f32.argtypes = [_i64p, _i64p, _u64, _f32p]
        L.hb_ref_open.restype = _int
        L.hb_ref_open.argtypes = [_i64p, _i64p, _u64, _int, _int, _i64p]
        _pp = ctypes.POINTER(_i64p)
        L.hb_ref_mp_opened_bits.restype = _u64
        L.hb_ref_mp_opened_bits.argtypes = [_int, _int, _int, _int, _u64]
        L.hb_ref_mp_eval_range.restype = _int
        L.hb_ref_mp_eval_range.argtypes = [_pp, _int, _u64, _u64, _int, _int, _u64, _int, _int, _pp]
        L.hb_ref_mp_eval_at.restype = _int
        L.hb_ref_mp_eval_at.argtypes = [_pp, _int, _u64p, _u64, _int, _int, _u64, _int, _int, _pp]
        _lib = L
    return _lib


def _as_i64(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint64:
        a = a.view(np.int64)
    if a.dtype != np.int64:
        raise TypeError("shares must be int64 or uint64 arrays, got %s" % a.dtype)
    return a.reshape(-1)


def _ptr(a, typ=_i64p):
    return a.ctypes.data_as(typ)


def mix64(z):
    return int(lib().hb_ref_mix64(_u64(z & (2**64 - 1))))


def sm(seed, j):
    return int(lib().hb_ref_sm(_u64(seed & (2**64 - 1)), _u64(j)))


def sm_sequence(seed, count):
    """First `count` outputs obtained by stepping the generator one output at a time."""
    state = _u64(seed & (2**64 - 1))
    return [int(lib().hb_ref_sm_next(ctypes.byref(state))) for _ in range(count)]


def tensor_seed(root_seed, tensor_id):
    return int(lib().hb_ref_tensor_seed(_u64(root_seed & (2**64 - 1)), _u64(tensor_id)))


VARIANT_PER_GATE, VARIANT_SHARED_MASK = 0, 1


def opened_bits(relu, k, m, n, variant=0):
    return int(lib().hb_ref_opened_bits_v(int(bool(relu)), k, m, _u64(n), variant))


def and_gate(U0, U1, V0, V1, a0, a1, b0, b1, c0, mask):
    z0, z1 = _u64(), _u64()
    lib().hb_ref_and_gate(*[_u64(v) for v in (U0, U1, V0, V1, a0, a1, b0, b1, c0, mask)],
                          ctypes.byref(z0), ctypes.byref(z1))
    return int(z0.value), int(z1.value)


def evaluate(share0, share1, k, m, seed, what, ring_bits=64, first=0, threads=1, variant=0):
    """Run the protocol on a whole array; returns the two share arrays selected by `what`.

    threads > 1 splits the element range into contiguous chunks evaluated by a thread pool
    (the C routine takes the global index of its first element, so results do not change).
    """
    s0, s1 = _as_i64(share0), _as_i64(share1)
    n = s0.size
    if s1.size != n:
        raise ValueError("share arrays differ in length")
    o0 = np.empty(n, dtype=np.int64)
    o1 = np.empty(n, dtype=np.int64)
    L = lib()

    def run(lo, hi):
        st = L.hb_ref_eval_range_v(_ptr(s0[lo:hi]), _ptr(s1[lo:hi]), _u64(first + lo), _u64(hi - lo), k, m,
                                   _u64(seed & (2**64 - 1)), ring_bits, variant, what,
                                   _ptr(o0[lo:hi]), _ptr(o1[lo:hi]))
        if st != 0:
            raise ValueError("oracle rejected arguments (status %d)" % st)

    threads = max(1, int(threads))
    if threads == 1 or n < 4096:
        # n == 0 still validates the arguments
        if n == 0:
            st = L.hb_ref_eval_range_v(None, None, _u64(first), _u64(0), k, m, _u64(seed & (2**64 - 1)),
                                       ring_bits, variant, what, None, None)
            if st != 0:
                raise ValueError("oracle rejected arguments (status %d)" % st)
        else:
            run(0, n)
    else:
        bounds = np.linspace(0, n, threads + 1).astype(np.int64)
        with ThreadPoolExecutor(max_workers=threads) as pool:
            list(pool.map(lambda ab: run(int(ab[0]), int(ab[1])), zip(bounds[:-1], bounds[1:])))
    return o0, o1


def evaluate_at(share0, share1, index, k, m, seed, what, ring_bits=64, variant=0):
    """Scattered elements: element index[i] of the tensor has share values share0[i], share1[i]."""
    s0, s1 = _as_i64(share0), _as_i64(share1)
    idx = np.ascontiguousarray(index, dtype=np.uint64).reshape(-1)
    if not (s0.size == s1.size == idx.size):
        raise ValueError("length mismatch")
    o0 = np.empty(idx.size, dtype=np.int64)
    o1 = np.empty(idx.size, dtype=np.int64)
    st = lib().hb_ref_eval_at_v(_ptr(s0), _ptr(s1), _ptr(idx, _u64p), _u64(idx.size), k, m,
                                _u64(seed & (2**64 - 1)), ring_bits, variant, what, _ptr(o0), _ptr(o1))
    if st != 0:
        raise ValueError("oracle rejected arguments (status %d)" % st)
    return o0, o1


def drelu(share0, share1, k, m, seed, ring_bits=64, threads=1, variant=0):
    o0, o1 = evaluate(share0, share1, k, m, seed, WHAT_DRELU, ring_bits, threads=threads, variant=variant)
    return o0, o1, opened_bits(False, k, m, o0.size, variant)


def relu(share0, share1, k, m, seed, ring_bits=64, threads=1, variant=0):
    o0, o1 = evaluate(share0, share1, k, m, seed, WHAT_RELU, ring_bits, threads=threads, variant=variant)
    return o0, o1, opened_bits(True, k, m, o0.size, variant)


def open_shares(share0, share1, binary=False, ring_bits=64):
    s0, s1 = _as_i64(share0), _as_i64(share1)
    out = np.empty(s0.size, dtype=np.int64)
    st = lib().hb_ref_open(_ptr(s0), _ptr(s1), _u64(s0.size), int(bool(binary)), ring_bits, _ptr(out))
    if st != 0:
        raise ValueError("oracle rejected arguments (status %d)" % st)
    return out


def eco_scan(share0, share1, seed=1, ring_bits=64, threads=1):
    """counts[m-1] = elements whose DReLU on [0, m) differs from the full ring, by running the protocol for every m.

    threads > 1 scans disjoint element ranges in a thread pool and adds the counts (a count is a sum over
    elements of a per-element comparison of reconstructed values, which do not depend on the element's index).
    """
    s0, s1 = _as_i64(share0), _as_i64(share1)
    n = s0.size

    def run(lo, hi):
        counts = np.zeros(64, dtype=np.uint64)
        st = lib().hb_ref_eco_scan(_ptr(s0[lo:hi]), _ptr(s1[lo:hi]), _u64(hi - lo), _u64(seed), ring_bits,
                                   _ptr(counts, _u64p))
        if st != 0:
            raise ValueError("oracle rejected arguments (status %d)" % st)
        return counts

    threads = max(1, int(threads))
    if threads == 1 or n < 4096:
        return run(0, n)
    bounds = np.linspace(0, n, threads + 1).astype(np.int64)
    with ThreadPoolExecutor(max_workers=threads) as pool:
        parts = list(pool.map(lambda ab: run(int(ab[0]), int(ab[1])), zip(bounds[:-1], bounds[1:])))
    return np.sum(np.stack(parts), axis=0, dtype=np.uint64)


def eco_choose(counts, ring_bits=64):
    c = np.ascontiguousarray(counts, dtype=np.uint64)
    return int(lib().hb_ref_eco_choose(_ptr(c, _u64p), ring_bits))


def wire_words(n, k, m, variant=0):
    return int(lib().hb_ref_wire_words_v(_u64(n), k, m, variant))


def relu_wire(share0, share1, k, m, seed, variant=0):
    """The packed words each party sends during one ReLU: (wire0, wire1) as uint64 arrays (layout in hb_ref.c)."""
    s0, s1 = _as_i64(share0), _as_i64(share1)
    words = wire_words(s0.size, k, m, variant)
    w0 = np.zeros(words, dtype=np.uint64)
    w1 = np.zeros(words, dtype=np.uint64)
    st = lib().hb_ref_relu_wire_v(_ptr(s0), _ptr(s1), _u64(s0.size), k, m, _u64(seed & (2**64 - 1)), variant,
                                  _ptr(w0, _u64p), _ptr(w1, _u64p))
    if st != 0:
        raise ValueError("oracle rejected arguments (status %d)" % st)
    return w0, w1


def share_f32(x, share_seed):
    """Encode float32 to 2^16 fixed point and share: share0 = generator outputs, share1 = x_fixed - share0."""
    xf = np.ascontiguousarray(x, dtype=np.float32).reshape(-1)
    s0 = np.empty(xf.size, dtype=np.int64)
    s1 = np.empty(xf.size, dtype=np.int64)
    st = lib().hb_ref_share_f32(xf.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), _u64(xf.size),
                                _u64(share_seed & (2**64 - 1)), _ptr(s0), _ptr(s1))
    if st != 0:
        raise ValueError("oracle rejected arguments (status %d)" % st)
    return s0, s1


def reveal_f32(share0, share1):
    s0, s1 = _as_i64(share0), _as_i64(share1)
    y = np.empty(s0.size, dtype=np.float32)
    st = lib().hb_ref_reveal_f32(_ptr(s0), _ptr(s1), _u64(s0.size), y.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    if st != 0:
        raise ValueError("oracle rejected arguments (status %d)" % st)
    return y


def sim_relu_f32(x, k, m, seed, share_seed, threads=1):
    """The simulator layer: share the floats, run the ReLU protocol, reveal."""
    s0, s1 = share_f32(x, share_seed)
    r0, r1, _ = relu(s0, s1, k, m, seed, threads=threads)
    return reveal_f32(r0, r1)


# ---- p >= 2 parties (oracle/hb_ref_mp.c) ------------------------------------------------------------------

def mp_opened_bits(relu, parties, k, m, n):
    """Bits one party sends to one other party."""
    return int(lib().hb_ref_mp_opened_bits(int(bool(relu)), parties, k, m, _u64(n)))


def _pointer_table(arrays, lo=0, hi=None):
    tab = (_i64p * len(arrays))()
    for q, a in enumerate(arrays):
        tab[q] = _ptr(a[lo:hi])
    return tab


def mp_evaluate(shares, k, m, seed, what, ring_bits=64, first=0, threads=1):
    """The protocol among len(shares) parties on whole arrays; returns the list of per-party arrays chosen by `what`."""
    sh = [_as_i64(a) for a in shares]
    p, n = len(sh), sh[0].size
    if any(a.size != n for a in sh):
        raise ValueError("share arrays differ in length")
    outs = [np.empty(n, dtype=np.int64) for _ in range(p)]
    L = lib()

    def run(lo, hi):
        st = L.hb_ref_mp_eval_range(_pointer_table(sh, lo, hi), p, _u64(first + lo), _u64(hi - lo), k, m,
                                    _u64(seed & (2**64 - 1)), ring_bits, what, _pointer_table(outs, lo, hi))
        if st != 0:
            raise ValueError("oracle rejected arguments (status %d)" % st)

    threads = max(1, int(threads))
    if threads == 1 or n < 4096:
        run(0, n)
    else:
        bounds = np.linspace(0, n, threads + 1).astype(np.int64)
        with ThreadPoolExecutor(max_workers=threads) as pool:
            list(pool.map(lambda ab: run(int(ab[0]), int(ab[1])), zip(bounds[:-1], bounds[1:])))
    return outs


def mp_evaluate_at(shares, index, k, m, seed, what, ring_bits=64):
    sh = [_as_i64(a) for a in shares]
    idx = np.ascontiguousarray(index, dtype=np.uint64).reshape(-1)
    if any(a.size != idx.size for a in sh):
        raise ValueError("length mismatch")
    outs = [np.empty(idx.size, dtype=np.int64) for _ in range(len(sh))]
    st = lib().hb_ref_mp_eval_at(_pointer_table(sh), len(sh), _ptr(idx, _u64p), _u64(idx.size), k, m,
                                 _u64(seed & (2**64 - 1)), ring_bits, what, _pointer_table(outs))
    if st != 0:
        raise ValueError("oracle rejected arguments (status %d)" % st)
    return outs


def mp_drelu(shares, k, m, seed, ring_bits=64, threads=1):
    outs = mp_evaluate(shares, k, m, seed, WHAT_DRELU, ring_bits, threads=threads)
    return outs, mp_opened_bits(False, len(outs), k, m, outs[0].size)


def mp_relu(shares, k, m, seed, ring_bits=64, threads=1):
    outs = mp_evaluate(shares, k, m, seed, WHAT_RELU, ring_bits, threads=threads)
    return outs, mp_opened_bits(True, len(outs), k, m, outs[0].size)
