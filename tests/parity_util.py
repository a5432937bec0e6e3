"""Whole-tensor comparison of device results with the CPU oracle, in host chunks.

The oracle evaluates any contiguous element range given the global index of its first element, so a tensor
of any size is compared element by element, chunk after chunk, with bounded host memory.  Everything is
integer: the comparison is `np.array_equal`, tolerance zero.
"""
import os

import numpy as np

import oracle

CHUNK = 1 << 26
THREADS = max(1, min(16, len(os.sched_getaffinity(0))))


def host(t):
    return t.cpu().numpy()


def assert_matches_oracle(s0, s1, outs, k, m, seed, what, variant=0, label=None, lo=0, hi=None):
    """outs = (out0, out1): device tensors holding what the library returned for the device shares (s0, s1).
    Every element of [lo, hi) is compared with oracle.evaluate on the same shares."""
    n = s0.numel()
    hi = n if hi is None else hi
    for a in range(lo, hi, CHUNK):
        b = min(a + CHUNK, hi)
        e0, e1 = oracle.evaluate(host(s0[a:b]), host(s1[a:b]), k, m, seed, what, first=a, threads=THREADS,
                                 variant=variant)
        g0, g1 = host(outs[0][a:b]), host(outs[1][a:b])
        if not (np.array_equal(g0, e0) and np.array_equal(g1, e1)):
            bad = np.nonzero((g0 != e0) | (g1 != e1))[0]
            raise AssertionError("%s: %d of %d elements differ from the oracle in [%d, %d); first at %d"
                                 % (label, bad.size, b - a, a, b, a + int(bad[0])))


def assert_mp_matches_oracle(shares, outs, k, m, seed, what, label=None):
    """The same for p parties: shares / outs are lists of device tensors."""
    n = shares[0].numel()
    for a in range(0, n, CHUNK):
        b = min(a + CHUNK, n)
        exp = oracle.mp_evaluate([host(s[a:b]) for s in shares], k, m, seed, what, first=a, threads=THREADS)
        for q, e in enumerate(exp):
            g = host(outs[q][a:b])
            if not np.array_equal(g, e):
                bad = np.nonzero(g != e)[0]
                raise AssertionError("%s: party %d, %d elements differ in [%d, %d); first at %d"
                                     % (label, q, bad.size, a, b, a + int(bad[0])))
