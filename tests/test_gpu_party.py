"""GPU parity of the party-faithful path (hb_relu_party): result shares AND every word each party puts on its wire
against the oracle's transcript -- bit for bit -- and result shares against the fused kernels at a larger size."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2309_04875_amd import hb

pytestmark = pytest.mark.gpu
DEV = "cuda"
SEED = 0x2309048750000001


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _rand_shares(rng, n):
    return (rng.integers(0, 1 << 64, n, dtype=np.uint64).view(np.int64),
            rng.integers(0, 1 << 64, n, dtype=np.uint64).view(np.int64))


@pytest.mark.parametrize("k,m", [(12, 20), (0, 64), (8, 14), (8, 18), (3, 4), (0, 2), (5, 12), (20, 53), (8, 12),
                                 (0, 33), (8, 24), (2, 5), (30, 62), (7, 16)])
def test_party_path_matches_oracle_shares_and_wire(k, m):
    w = m - k
    L = min(64 // w, 32)
    rng = np.random.default_rng(k * 64 + m)
    i64 = np.iinfo(np.int64)
    for n in sorted({1, max(1, L - 1), L, L + 1, 64, 65, 100, 4096 + 17}):
        s0, s1 = _rand_shares(rng, n)
        s0[0], s1[0] = i64.min, i64.max
        seed = SEED + n
        o0, o1, w0, w1, wire_bytes = hb.hb_relu_party(_dev(s0), _dev(s1), k, m, seed)
        e0, e1, _ = oracle.relu(s0, s1, k, m, seed)
        assert np.array_equal(o0.cpu().numpy(), e0) and np.array_equal(o1.cpu().numpy(), e1), (k, m, n)
        x0, x1 = oracle.relu_wire(s0, s1, k, m, seed)
        assert wire_bytes == 8 * x0.size == 8 * oracle.wire_words(n, k, m)
        assert np.array_equal(w0.cpu().numpy().view(np.uint64), x0), (k, m, n)
        assert np.array_equal(w1.cpu().numpy().view(np.uint64), x1), (k, m, n)


@pytest.mark.parametrize("k,m", [(12, 20), (0, 64), (8, 14), (8, 18), (3, 4), (0, 2), (5, 12), (20, 53), (8, 12),
                                 (0, 33), (8, 24), (2, 5), (30, 62), (7, 16)])
def test_party_path_on_the_shared_mask_layout_matches_oracle_shares_and_wire(k, m):
    """One mask of P per round: three wire words per round and group; shares and wire against the oracle's variant 1."""
    w = m - k
    L = min(64 // w, 32)
    SH = hb.HB_DEALER_SHARED_MASK
    rng = np.random.default_rng(1000 + k * 64 + m)
    for n in sorted({1, max(1, L - 1), L, L + 1, 64, 65, 100, 4096 + 17}):
        s0, s1 = _rand_shares(rng, n)
        seed = SEED + 3 * n
        o0, o1, w0, w1, wire_bytes = hb.hb_relu_party_ex(_dev(s0), _dev(s1), k, m, seed, SH)
        e0, e1, _ = oracle.relu(s0, s1, k, m, seed, variant=1)
        assert np.array_equal(o0.cpu().numpy(), e0) and np.array_equal(o1.cpu().numpy(), e1), (k, m, n)
        x0, x1 = oracle.relu_wire(s0, s1, k, m, seed, variant=1)
        assert wire_bytes == 8 * x0.size == 8 * oracle.wire_words(n, k, m, 1) == 8 * hb.hb_party_wire_words_ex(n, k, m, SH)
        assert np.array_equal(w0.cpu().numpy().view(np.uint64), x0), (k, m, n)
        assert np.array_equal(w1.cpu().numpy().view(np.uint64), x1), (k, m, n)
    # the standard layout through the _ex entry point is hb_relu_party bit for bit
    s0, s1 = _rand_shares(rng, 1000)
    a = hb.hb_relu_party_ex(_dev(s0), _dev(s1), k, m, SEED, hb.HB_DEALER_PER_GATE)
    b = hb.hb_relu_party(_dev(s0), _dev(s1), k, m, SEED)
    assert all(torch.equal(x, y) for x, y in zip(a[:4], b[:4])) and a[4] == b[4]


def test_shared_mask_wire_is_the_opened_bit_count_at_size():
    """2^21 elements: the bytes each party writes are exactly the opened bits of the layout (w * L = 64, 64 | n):
    217 instead of 241 bits per element at w = 8."""
    n = 1 << 21
    g = torch.Generator(device=DEV)
    g.manual_seed(5)
    s0 = torch.randint(-2**62, 2**62, (n,), generator=g, device=DEV, dtype=torch.int64)
    s1 = torch.randint(-2**62, 2**62, (n,), generator=g, device=DEV, dtype=torch.int64)
    SH = hb.HB_DEALER_SHARED_MASK
    for (k, m) in [(12, 20), (0, 64), (8, 24)]:
        r0, r1, bits = hb.hb_relu_ex(s0, s1, k, m, SEED, SH)
        o0, o1, w0, w1, wire_bytes = hb.hb_relu_party_ex(s0, s1, k, m, SEED, SH)
        assert torch.equal(o0, r0) and torch.equal(o1, r1)
        assert 8 * wire_bytes == bits == hb.hb_opened_bits_ex(True, k, m, n, SH)
    assert hb.hb_opened_bits_ex(True, 12, 20, 1, SH) == 217
    assert hb.hb_party_wire_words_ex(n, 12, 20, 7) == 0 and hb.hb_party_workspace_bytes_ex(n, 12, 20, 7) == 0
    with pytest.raises(hb.HbError):
        hb.hb_relu_party_ex(s0[:64], s1[:64], 12, 20, SEED, 7, workspace=torch.empty(1 << 16, dtype=torch.uint8, device=DEV))


@pytest.mark.parametrize("k,m", [(12, 20), (8, 14), (0, 64)])
def test_party_path_equals_fused_kernels_at_size(k, m):
    n = 1 << 21
    g = torch.Generator(device=DEV)
    g.manual_seed(k + m)
    s0 = torch.randint(-2**62, 2**62, (n,), generator=g, device=DEV, dtype=torch.int64)
    s1 = torch.randint(-2**62, 2**62, (n,), generator=g, device=DEV, dtype=torch.int64)
    r0, r1, bits = hb.hb_relu(s0, s1, k, m, SEED)
    o0, o1, w0, w1, wire_bytes = hb.hb_relu_party(s0, s1, k, m, SEED)
    assert torch.equal(o0, r0) and torch.equal(o1, r1)
    w = m - k
    if 64 % w == 0:
        assert 8 * wire_bytes == bits               # every wire bit is an opened bit
    else:
        assert 8 * wire_bytes > bits
    # the opened multiply values add up to x - a and DReLU - b for some dealer (a, b): reconstructing through the
    # wire must give the same product as the shares do
    assert torch.equal(o0 + o1, r0 + r1)


def test_party_path_argument_errors():
    n = 1000
    t = [torch.zeros(n, dtype=torch.int64, device=DEV) for _ in range(4)]
    need = hb.hb_party_workspace_bytes(n, 12, 20)
    assert need > 0 and hb.hb_party_workspace_bytes(n, 20, 12) == 0
    ws = torch.empty(need + 512, dtype=torch.uint8, device=DEV)
    base = ws.data_ptr()
    off = (-base) % 256
    p = [x.data_ptr() for x in t]
    call = lambda *a: hb.raw("hb_relu_party", *a)
    wb = ctypes.c_uint64(0)
    assert call(p[0], p[1], n, 12, 20, SEED, p[2], p[3], base + off, need, ctypes.byref(wb), None) == hb.HB_OK
    assert wb.value == 8 * hb.hb_party_wire_words(n, 12, 20)
    assert call(p[0], p[1], n, 12, 20, SEED, p[2], p[3], base + off, need - 1, None, None) == hb.HB_EINVAL
    assert call(p[0], p[1], n, 12, 20, SEED, p[2], p[3], None, need, None, None) == hb.HB_EINVAL
    assert call(p[0], p[1], n, 12, 20, SEED, p[2], p[3], base + off + 8, need, None, None) == hb.HB_EALIGN
    assert call(p[0], p[1], n, 12, 20, SEED, p[0], p[3], base + off, need, None, None) == hb.HB_EINVAL   # in place
    assert call(p[0], p[1], n, 20, 12, SEED, p[2], p[3], base + off, need, None, None) == hb.HB_EINVAL
    assert call(None, None, 0, 12, 20, SEED, None, None, None, 0, ctypes.byref(wb), None) == hb.HB_OK and wb.value == 0
    torch.cuda.synchronize()
