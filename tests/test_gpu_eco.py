"""GPU parity of the zero-error high-cut scan (hb_eco_scan) against the oracle, which runs the protocol at
every cut, and -- at sizes the oracle cannot reach -- against the property the oracle's pins establish:
counts[m-1] = number of elements whose bit m-1 differs from the sign bit.  Integer counts: tolerance 0."""
import numpy as np
import pytest
import torch

import oracle
from paper_2309_04875_amd import hb, workloads
from parity_util import THREADS, host

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _shares(x, rng):
    s0 = rng.integers(0, 1 << 64, x.size, dtype=np.uint64)
    return s0.view(np.int64), (x.view(np.uint64) - s0).view(np.int64)


def _bit_counts_torch(x):
    d = x ^ (x >> 63)
    return torch.stack([((d >> b) & 1).sum() for b in range(64)])


@pytest.mark.parametrize("n", [1, 2, 63, 64, 65, 4095, 4096, 4097, 20000])
def test_eco_scan_matches_protocol_oracle(n):
    rng = np.random.default_rng(n)
    x = np.rint(rng.standard_normal(n) * 3 * 65536).astype(np.int64)
    x[: min(n, 3)] = np.array([np.iinfo(np.int64).min, -1, np.iinfo(np.int64).max])[: min(n, 3)]
    s0, s1 = _shares(x, rng)
    got = hb.hb_eco_scan(_dev(s0), _dev(s1)).cpu().numpy().view(np.uint64)
    exp = oracle.eco_scan(s0, s1)
    assert np.array_equal(got, exp)
    assert hb.hb_eco_choose(got) == oracle.eco_choose(exp)


def test_eco_scan_uniform_shares_unaligned_and_empty():
    rng = np.random.default_rng(5)
    n = 300001
    s0 = rng.integers(0, 1 << 64, n + 1, dtype=np.uint64).view(np.int64)
    s1 = rng.integers(0, 1 << 64, n + 1, dtype=np.uint64).view(np.int64)
    d0, d1 = _dev(s0)[1:], _dev(s1)[1:]
    assert d0.data_ptr() % 16 == 8
    got = hb.hb_eco_scan(d0, d1)
    assert torch.equal(got, _bit_counts_torch(d0 + d1))
    assert int(got[62]) > n // 3                      # uniform x: about half of the elements disagree at every bit
    e = torch.empty(0, dtype=torch.int64, device=DEV)
    c = torch.full((64,), 7, dtype=torch.int64, device=DEV)
    hb.hb_eco_scan(e, e, c)
    assert int(c.abs().sum()) == 0
    with pytest.raises(hb.HbError):
        hb.hb_eco_scan(d0, d1, d0[:64])               # counts inside an input


def test_eco_scan_many_blocks_matches_protocol_oracle():
    """2^22 + 7 elements (every block of the launch takes several chunks): all 64 counts against the oracle,
    which evaluates the protocol at every cut for every element."""
    spec = workloads.resnet18_cifar_batch512()[0]
    x, s0, s1 = workloads.materialize_on_device(spec, DEV)
    n = (1 << 22) + 7
    got = hb.hb_eco_scan(s0[:n], s1[:n]).cpu().numpy().view(np.uint64)
    exp = oracle.eco_scan(host(s0[:n]), host(s1[:n]), threads=THREADS)
    assert np.array_equal(got, exp)
    assert hb.hb_eco_choose(got) == oracle.eco_choose(exp)


def test_eco_scan_full_size_tensor_and_choice():
    """Largest tensor of the batch-512 set (2^25 elements; the protocol oracle needs 128 evaluations per element,
    about a minute of host time at this size): every count against the bit test of Theorem 1 on the device, the
    property the oracle's pins establish; the oracle itself is compared at 2^22 elements above."""
    spec = workloads.resnet18_cifar_batch512()[0]
    x, s0, s1 = workloads.materialize_on_device(spec, DEV)
    got = hb.hb_eco_scan(s0, s1)
    assert torch.equal(got, _bit_counts_torch(x))
    m = hb.hb_eco_choose(got)
    # zero-error cut: every |x| fits in m bits, and not in m - 1
    amax = int(torch.maximum(x, -x - 1).max())        # max of x (x >= 0) and -x-1 (x < 0)
    assert amax < (1 << (m - 1)) and amax >= (1 << (m - 2))
    d0, d1, _ = hb.hb_drelu(s0, s1, 0, m, 99)
    assert torch.equal(d0 + d1, (x >= 0).to(torch.int64))
