"""GPU parity of hb_relu_mp / hb_drelu_mp (3 and 4 parties) against the p-party oracle, bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2309_04875_amd import hb, workloads
from parity_util import assert_mp_matches_oracle

pytestmark = pytest.mark.gpu

SEED = 0x2309048750000033
DEV = "cuda"


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _host(t):
    return t.cpu().numpy()


def _rand(rng, p, n):
    return [rng.integers(0, 1 << 64, n, dtype=np.uint64).view(np.int64) for _ in range(p)]


def _check(shares, k, m, seed):
    p, n = len(shares), shares[0].size
    d = [_dev(s) for s in shares]
    got, bits = hb.hb_relu_mp(d, k, m, seed)
    exp, ebits = oracle.mp_relu(shares, k, m, seed)
    for q in range(p):
        assert np.array_equal(_host(got[q]), exp[q]), ("relu", p, q, k, m, n)
    assert bits == ebits == hb.hb_opened_bits_mp(True, p, k, m, n)
    got, bits = hb.hb_drelu_mp(d, k, m, seed)
    exp, ebits = oracle.mp_drelu(shares, k, m, seed)
    for q in range(p):
        assert np.array_equal(_host(got[q]), exp[q]), ("drelu", p, q, k, m, n)
    assert bits == ebits == hb.hb_opened_bits_mp(False, p, k, m, n)


@pytest.mark.parametrize("p", [3, 4])
@pytest.mark.parametrize("w", range(1, 65))
def test_every_width(p, w):
    rng = np.random.default_rng(1000 * p + w)
    L = min(64 // w, 64 // p)
    n = 2 * 256 * L + L // 2 + 1           # thread blocks / tiles of groups and a partial group
    for k in sorted({0, 64 - w}):
        _check(_rand(rng, p, n), k, k + w, SEED ^ (w * 40503))


@pytest.mark.parametrize("p", [3, 4])
@pytest.mark.parametrize("k,m", [(12, 20), (0, 64), (8, 14), (8, 18), (3, 4), (0, 2), (8, 13), (2, 34)])
def test_ragged_sizes_extremes_and_alignment(p, k, m):
    w = m - k
    L = min(64 // w, 64 // p)
    i64 = np.iinfo(np.int64)
    rng = np.random.default_rng(p * 4096 + k * 64 + m)
    for n in sorted({1, 2, L - 1, L, L + 1, 64 * L - 1, 64 * L, 64 * L + 1, 257 * L + 3, 1000} - {0}):
        s = _rand(rng, p, n)
        ext = np.array([0, -1, i64.min, i64.max, 1, i64.min + 1], dtype=np.int64)
        c = min(n, ext.size)
        for q in range(p):
            s[q][:c] = np.roll(ext, q)[:c]
        _check(s, k, m, SEED + n)
    # buffers that are only 8-byte aligned take the thread-per-group kernel
    s = _rand(rng, p, 3001)
    d = [_dev(a)[1:] for a in s]
    got, _ = hb.hb_relu_mp(d, k, m, SEED)
    exp, _ = oracle.mp_relu([a[1:] for a in s], k, m, SEED)
    for q in range(p):
        assert np.array_equal(_host(got[q]), exp[q])


def test_two_parties_is_hb_relu():
    rng = np.random.default_rng(2)
    s = _rand(rng, 2, 5000)
    d = [_dev(a) for a in s]
    for (k, m) in [(12, 20), (0, 64), (0, 1)]:
        got, bits = hb.hb_relu_mp(d, k, m, SEED)
        r0, r1, rb = hb.hb_relu(d[0], d[1], k, m, SEED)
        assert torch.equal(got[0], r0) and torch.equal(got[1], r1) and bits == rb
        got, bits = hb.hb_drelu_mp(d, k, m, SEED)
        r0, r1, rb = hb.hb_drelu(d[0], d[1], k, m, SEED)
        assert torch.equal(got[0], r0) and torch.equal(got[1], r1) and bits == rb


@pytest.mark.parametrize("p", [3, 4])
def test_in_place_and_reconstruction(p):
    """Outputs written over the inputs; the opened result is max(x, 0) inside the window of correctness."""
    rng = np.random.default_rng(70 + p)
    k, m = 12, 22
    n = 100003
    x = np.rint(rng.standard_normal(n) * 2 * 65536).astype(np.int64)
    sh = [rng.integers(0, 1 << 64, n, dtype=np.uint64) for _ in range(p - 1)]
    last = x.view(np.uint64).copy()
    for a in sh:
        last -= a
    shares = [a.view(np.int64) for a in sh] + [last.view(np.int64)]
    exp, _ = oracle.mp_relu(shares, k, m, SEED)
    d = [_dev(a) for a in shares]
    got, _ = hb.hb_relu_mp(d, k, m, SEED, outs=d)
    tot = np.zeros(n, dtype=np.int64)
    for q in range(p):
        assert got[q].data_ptr() == d[q].data_ptr()
        assert np.array_equal(_host(got[q]), exp[q])
        tot = tot + _host(got[q])
    ok = (np.abs(x) >= (p - 1) * (1 << k)) & (np.abs(x) < (1 << (m - 1)) - (p - 1) * (1 << k))
    assert np.array_equal(tot[ok], np.maximum(x, 0)[ok])


@pytest.mark.parametrize("p", [3, 4])
def test_full_size_tensor_every_element(p):
    """One tensor of the batch-512 set (2^25 elements) shared p ways: every element of every party's output
    against the oracle; the reconstruction identity on the device as an extra check."""
    spec = workloads.resnet18_cifar_batch512()[0]
    x, s0, s1 = workloads.materialize_on_device(spec, DEV)
    n, k, m = spec.n, spec.k, spec.m
    g = torch.Generator(device=DEV)
    g.manual_seed(17 + p)
    extra = [torch.randint(-(1 << 62), 1 << 62, (n,), dtype=torch.int64, device=DEV, generator=g) for _ in range(p - 2)]
    shares = [s0, s1 - sum(extra)] + extra          # still sums to x (mod 2^64)
    got, bits = hb.hb_relu_mp(shares, k, m, SEED)
    assert bits == oracle.mp_opened_bits(True, p, k, m, n)
    assert_mp_matches_oracle(shares, got, k, m, SEED, oracle.WHAT_RELU, label=("relu_mp", p))
    w = m - k
    u = sum((s >> k) for s in shares) & ((1 << w) - 1)
    dexp = 1 - ((u >> (w - 1)) & 1)
    assert torch.equal(sum(got), x * dexp)
    got, bits = hb.hb_drelu_mp(shares, k, m, SEED)
    assert bits == oracle.mp_opened_bits(False, p, k, m, n)
    assert_mp_matches_oracle(shares, got, k, m, SEED, oracle.WHAT_DRELU, label=("drelu_mp", p))


def test_errors():
    z = [torch.zeros(64, dtype=torch.int64, device=DEV) for _ in range(3)]
    o = [torch.full((64,), 5, dtype=torch.int64, device=DEV) for _ in range(3)]
    with pytest.raises(hb.HbError) as err:
        hb.hb_relu_mp(z, 20, 12, 1, outs=o)                       # bad slice
    assert err.value.status == hb.HB_EINVAL
    with pytest.raises(hb.HbError):
        hb.hb_relu_mp(z[:1], 12, 20, 1, outs=o[:1])               # one party
    five = z + [torch.zeros(64, dtype=torch.int64, device=DEV) for _ in range(2)]
    with pytest.raises(hb.HbError):
        hb.hb_relu_mp(five, 12, 20, 1)                            # more parties than the library supports
    with pytest.raises(hb.HbError):
        hb.hb_relu_mp(z, 12, 20, 1, outs=[o[0], o[0], o[2]])      # two outputs are the same buffer
    buf = torch.zeros(100, dtype=torch.int64, device=DEV)
    with pytest.raises(hb.HbError):
        hb.hb_relu_mp(z, 12, 20, 1, outs=[buf[0:64], buf[32:96], o[2]])   # outputs overlap partially
    assert hb.hb_opened_bits_mp(True, 5, 12, 20, 1) == 0 and hb.hb_opened_bits_mp(True, 3, 20, 12, 1) == 0
    torch.cuda.synchronize()
    assert all(int(t.min()) == 5 and int(t.max()) == 5 for t in o)        # nothing was written
    e = [torch.zeros(0, dtype=torch.int64, device=DEV) for _ in range(3)]
    outs, bits = hb.hb_relu_mp(e, 12, 20, 1)
    assert bits == 0 and all(t.numel() == 0 for t in outs)
