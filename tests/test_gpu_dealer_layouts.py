"""GPU parity of the shared-mask dealer layout (hb_*_ex with HB_DEALER_SHARED_MASK) against the oracle's
variant 1, bit for bit, and of HB_DEALER_PER_GATE against the plain entry points.
"""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2309_04875_amd import hb, workloads
from parity_util import assert_matches_oracle

pytestmark = pytest.mark.gpu

SEED = 0x2309048750000077
DEV = "cuda"
SHARED = hb.HB_DEALER_SHARED_MASK


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _host(t):
    return t.cpu().numpy()


def _rand_shares(rng, n):
    return (rng.integers(0, 1 << 64, n, dtype=np.uint64).view(np.int64),
            rng.integers(0, 1 << 64, n, dtype=np.uint64).view(np.int64))


def _check(s0, s1, k, m, seed):
    d0, d1 = _dev(s0), _dev(s1)
    g0, g1, bits = hb.hb_relu_ex(d0, d1, k, m, seed, SHARED)
    e0, e1, ebits = oracle.relu(s0, s1, k, m, seed, variant=oracle.VARIANT_SHARED_MASK)
    assert np.array_equal(_host(g0), e0) and np.array_equal(_host(g1), e1), ("relu", k, m, s0.size)
    assert bits == ebits == hb.hb_opened_bits_ex(True, k, m, s0.size, SHARED)
    g0, g1, bits = hb.hb_drelu_ex(d0, d1, k, m, seed, SHARED)
    e0, e1, ebits = oracle.drelu(s0, s1, k, m, seed, variant=oracle.VARIANT_SHARED_MASK)
    assert np.array_equal(_host(g0), e0) and np.array_equal(_host(g1), e1), ("drelu", k, m, s0.size)
    assert bits == ebits == hb.hb_opened_bits_ex(False, k, m, s0.size, SHARED)


@pytest.mark.parametrize("w", range(1, 65))
def test_every_width_shared_mask(w):
    rng = np.random.default_rng(500 + w)
    L = min(64 // w, 32)
    n = 3 * 256 * L + L // 2 + 1           # several tiles / thread blocks of groups and a partial group
    for k in sorted({0, 64 - w}):
        s0, s1 = _rand_shares(rng, n)
        _check(s0, s1, k, k + w, SEED ^ (w * 2654435761))


@pytest.mark.parametrize("k,m", [(12, 20), (0, 64), (8, 14), (8, 18), (3, 4), (0, 2)])
def test_ragged_sizes_shared_mask(k, m):
    w = m - k
    L = min(64 // w, 32)
    i64 = np.iinfo(np.int64)
    rng = np.random.default_rng(k * 64 + m + 7)
    for n in sorted({1, L - 1, L, L + 1, 64 * L - 1, 64 * L + 1, 256 * L + 1, 1000} - {0}):
        s0, s1 = _rand_shares(rng, n)
        ext = np.array([0, -1, i64.min, i64.max, 1, i64.min + 1], dtype=np.int64)
        c = min(n, ext.size)
        s0[:c] = ext[:c]
        s1[:c] = ext[::-1][:c]
        _check(s0, s1, k, m, SEED + n)
    # only 8-byte aligned buffers take the thread-per-group kernel
    s0, s1 = _rand_shares(rng, 2001)
    d0, d1 = _dev(s0)[1:], _dev(s1)[1:]
    g0, g1, _ = hb.hb_relu_ex(d0, d1, k, m, SEED, SHARED)
    e0, e1, _ = oracle.relu(s0[1:], s1[1:], k, m, SEED, variant=1)
    assert np.array_equal(_host(g0), e0) and np.array_equal(_host(g1), e1)


def test_per_gate_layout_is_the_plain_entry_point():
    rng = np.random.default_rng(12)
    for (k, m) in [(12, 20), (0, 64), (8, 14), (0, 1)]:
        s0, s1 = _rand_shares(rng, 5000)
        d0, d1 = _dev(s0), _dev(s1)
        r0, r1, rb = hb.hb_relu(d0, d1, k, m, SEED)
        b0, b1, bb = hb.hb_relu_ex(d0, d1, k, m, SEED, hb.HB_DEALER_PER_GATE)
        assert torch.equal(r0, b0) and torch.equal(r1, b1) and rb == bb
        a0, a1, ab = hb.hb_drelu(d0, d1, k, m, SEED)
        b0, b1, bb = hb.hb_drelu_ex(d0, d1, k, m, SEED, hb.HB_DEALER_PER_GATE)
        assert torch.equal(a0, b0) and torch.equal(a1, b1) and ab == bb
        # the layouts differ in the shares, not in what they reconstruct to.  (The ReLU shares are even equal:
        # they depend on the DReLU shares only through the opened DReLU - b, i.e. through the reconstructed DReLU.)
        c0, c1, cb = hb.hb_relu_ex(d0, d1, k, m, SEED, SHARED)
        assert torch.equal(hb.hb_open(c0, c1), hb.hb_open(r0, r1))
        q0, q1, qb = hb.hb_drelu_ex(d0, d1, k, m, SEED, SHARED)
        assert torch.equal(hb.hb_open(q0, q1), hb.hb_open(a0, a1))
        if m - k > 1:
            assert not torch.equal(q0, a0)
            assert cb < rb and qb < ab


def test_batch_shared_mask_one_image_set_and_mixed():
    specs = list(workloads.resnet18_cifar())
    specs += [workloads.TensorSpec("mixed", 100 + i, (257 + 13 * i,), k, m, 2.0, "normal", 700 + i)
              for i, (k, m) in enumerate([(8, 14), (0, 64), (5, 12), (3, 4), (8, 18), (12, 20)])]
    for relu in (True, False):
        items, expect = [], []
        for spec in specs:
            x, s0, s1 = workloads.materialize(spec)
            seed = hb.hb_tensor_seed(SEED, spec.tensor_id)
            d0, d1 = _dev(s0), _dev(s1)
            items.append((d0, d1, torch.empty_like(d0), torch.empty_like(d1), spec.k, spec.m, seed))
            expect.append((oracle.relu if relu else oracle.drelu)(s0, s1, spec.k, spec.m, seed, variant=1))
        bits = (hb.hb_relu_batch_ex if relu else hb.hb_drelu_batch_ex)(items, SHARED)
        for (d0, d1, o0, o1, k, m, seed), (e0, e1, _) in zip(items, expect):
            assert np.array_equal(_host(o0), e0) and np.array_equal(_host(o1), e1), (k, m)
        assert bits == sum(e[2] for e in expect)


def test_full_size_shared_mask_every_element():
    """Three tensors of the batch-512 set at full size in one batched call on the shared-mask layout, and the
    largest one through the per-tensor entry points (ReLU and DReLU): every element against the oracle."""
    specs = workloads.resnet18_cifar_batch512()
    items, keep = [], []
    for spec in (specs[0], specs[7], specs[16]):
        x, s0, s1 = workloads.materialize_on_device(spec, DEV)
        seed = hb.hb_tensor_seed(SEED, spec.tensor_id)
        items.append((s0, s1, torch.empty_like(s0), torch.empty_like(s1), spec.k, spec.m, seed))
        keep.append((spec, x))
    bits = hb.hb_relu_batch_ex(items, SHARED)
    assert bits == sum(oracle.opened_bits(True, s.k, s.m, s.n, variant=1) for s, _ in keep)
    for (spec, x), (s0, s1, o0, o1, k, m, seed) in zip(keep, items):
        assert_matches_oracle(s0, s1, (o0, o1), k, m, seed, oracle.WHAT_RELU, variant=1, label=("shared batch", spec))
        w = m - k
        u = ((s0 >> k) + (s1 >> k)) & ((1 << w) - 1)
        dexp = 1 - ((u >> (w - 1)) & 1)
        assert torch.equal(hb.hb_open(o0, o1), x * dexp), spec
    s0, s1, o0, o1, k, m, seed = items[0]
    hb.hb_relu_ex(s0, s1, k, m, seed, SHARED, o0, o1)
    assert_matches_oracle(s0, s1, (o0, o1), k, m, seed, oracle.WHAT_RELU, variant=1, label="relu_ex shared")
    hb.hb_drelu_ex(s0, s1, k, m, seed, SHARED, o0, o1)
    assert_matches_oracle(s0, s1, (o0, o1), k, m, seed, oracle.WHAT_DRELU, variant=1, label="drelu_ex shared")


def test_unknown_layout_is_rejected():
    z = torch.zeros(64, dtype=torch.int64, device=DEV)
    o0, o1 = torch.full_like(z, 5), torch.full_like(z, 5)
    for bad in (2, -1, 7):
        with pytest.raises(hb.HbError) as err:
            hb.hb_relu_ex(z, z.clone(), 12, 20, 1, bad, o0, o1)
        assert err.value.status == hb.HB_EINVAL
        with pytest.raises(hb.HbError):
            hb.hb_drelu_batch_ex([(z, z.clone(), o0, o1, 12, 20, 1)], bad)
        assert hb.hb_opened_bits_ex(True, 12, 20, 1, bad) == 0
    torch.cuda.synchronize()
    assert int(o0.min()) == 5 and int(o1.max()) == 5       # nothing was written
