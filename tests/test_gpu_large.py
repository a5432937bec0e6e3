"""GPU parity beyond 2^31 elements: element, group and dealer-word indices that do not fit 32 bits.

One tensor of 2^31 + 2^20 + 77 int64 elements per share (17 GB each; four such buffers live on the device).
The wavefront-tile kernel at (12, 20) is compared with the oracle on EVERY element, chunk by chunk (about
20 s of oracle time on 16 host threads).  The full-ring and the 8-byte-aligned runs are compared with the
oracle on every element of the ranges where an index crosses a power of two (both ends, around element 2^31,
around group 2^28) and on random elements; the reconstruction identity is checked on every element.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2309_04875_amd import hb
from parity_util import assert_matches_oracle

pytestmark = pytest.mark.gpu

SEED = 0x2309048750000055
DEV = "cuda"
N = (1 << 31) + (1 << 20) + 77
CHUNK = 1 << 27
# element ranges compared in full where the whole tensor is not: the two ends, element 2^31, group 2^28 (L = 8)
REGIONS = [(0, 1 << 22), ((1 << 31) - (1 << 22), (1 << 31) + (1 << 22)), ((1 << 28) - (1 << 20), (1 << 28) + (1 << 20)),
           (N - (1 << 22), N)]


def _fill_random(t, gen):
    for lo in range(0, t.numel(), CHUNK):
        hi = min(lo + CHUNK, t.numel())
        t[lo:hi] = torch.randint(-(1 << 63), (1 << 63) - 1, (hi - lo,), dtype=torch.int64, device=DEV, generator=gen)


def _samples(rng):
    edge = np.concatenate([np.arange(0, 600), np.arange(N - 600, N),
                           np.arange((1 << 31) - 600, (1 << 31) + 600),
                           np.arange((1 << 28) - 20, (1 << 28) + 20)])       # group index 2^31 at L = 8
    return np.unique(np.concatenate([edge, rng.integers(0, N, 1 << 14)])).astype(np.int64)


def test_relu_beyond_2_pow_31_elements():
    free, _ = torch.cuda.mem_get_info()
    if free < 5 * 8 * N:
        pytest.skip("needs about 86 GB of free device memory")
    gen = torch.Generator(device=DEV)
    gen.manual_seed(2031)
    s0 = torch.empty(N, dtype=torch.int64, device=DEV)
    s1 = torch.empty(N, dtype=torch.int64, device=DEV)
    _fill_random(s0, gen)
    _fill_random(s1, gen)
    o0, o1 = torch.empty_like(s0), torch.empty_like(s1)
    rng = np.random.default_rng(31)
    idx = _samples(rng)
    tidx = torch.from_numpy(idx).to(DEV)
    h0, h1 = s0[tidx].cpu().numpy(), s1[tidx].cpu().numpy()

    for (k, m) in [(12, 20), (0, 64)]:        # wavefront-tile kernel, thread-per-group kernel with L = 1
        _, _, bits = hb.hb_relu(s0, s1, k, m, SEED, o0, o1)
        assert bits == oracle.opened_bits(True, k, m, N)
        e0, e1 = oracle.evaluate_at(h0, h1, idx.astype(np.uint64), k, m, SEED, oracle.WHAT_RELU)
        assert np.array_equal(o0[tidx].cpu().numpy(), e0) and np.array_equal(o1[tidx].cpu().numpy(), e1), (k, m)
        if (k, m) == (12, 20):
            assert_matches_oracle(s0, s1, (o0, o1), k, m, SEED, oracle.WHAT_RELU, label="2^31 + 2^20 + 77 elements")
        else:
            for (lo, hi) in REGIONS:
                assert_matches_oracle(s0, s1, (o0, o1), k, m, SEED, oracle.WHAT_RELU, label=(k, m), lo=lo, hi=hi)
        w = m - k
        for lo in range(0, N, CHUNK):
            hi = min(lo + CHUNK, N)
            a, b = s0[lo:hi], s1[lo:hi]
            if w == 64:
                dexp = ((a + b) >= 0).to(torch.int64)
            else:
                u = ((a >> k) + (b >> k)) & ((1 << w) - 1)
                dexp = 1 - ((u >> (w - 1)) & 1)
            assert torch.equal(o0[lo:hi] + o1[lo:hi], (a + b) * dexp), (k, m, lo)

    # buffers that are only 8-byte aligned: thread-per-group kernel at L = 8 (group index beyond 2^28, dealer word
    # index beyond 2^33)
    k, m = 12, 20
    hb.hb_relu(s0[1:], s1[1:], k, m, SEED, o0[1:], o1[1:])
    sub = idx[idx >= 1]
    tsub = torch.from_numpy(sub).to(DEV)
    e0, e1 = oracle.evaluate_at(s0[tsub].cpu().numpy(), s1[tsub].cpu().numpy(), (sub - 1).astype(np.uint64), k, m, SEED,
                                oracle.WHAT_RELU)
    assert np.array_equal(o0[tsub].cpu().numpy(), e0) and np.array_equal(o1[tsub].cpu().numpy(), e1)

    # reconstruction over the whole range
    out = hb.hb_open(o0[1:], o1[1:], False, out=o0[1:])
    for lo in range(1, N, CHUNK):
        hi = min(lo + CHUNK, N)
        a, b = s0[lo:hi], s1[lo:hi]
        u = ((a >> k) + (b >> k)) & 255
        assert torch.equal(out[lo - 1:hi - 1], (a + b) * (1 - (u >> 7))), lo
