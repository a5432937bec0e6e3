"""GPU parity of the float boundary (hb_share_f32, hb_reveal_f32) and of the one-kernel simulator
(hb_sim_relu_f32) against the oracle.  Shares are integers (tolerance 0); the floats are results of a fixed
sequence of IEEE operations (int64 -> double, scale by 2^-16, -> float), so they are compared bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2309_04875_amd import hb
from parity_util import THREADS

pytestmark = pytest.mark.gpu
DEV = "cuda"
SEED = 0x2309048750000001


def _bits(a):
    return np.asarray(a, dtype=np.float32).view(np.uint32)


def _inputs(rng, n):
    x = (rng.standard_normal(n) * 2).astype(np.float32)
    sp = np.array([0.0, -0.0, 1.5 / 65536, 2.5 / 65536, -2.5 / 65536, np.nan, np.inf, -np.inf, 3e38, -3e38, 2.0 ** 24],
                  dtype=np.float32)
    c = min(n, sp.size)
    x[:c] = sp[:c]
    return x


@pytest.mark.parametrize("n", [1, 2, 3, 511, 512, 513, 70001])
def test_share_and_reveal_match_oracle(n):
    rng = np.random.default_rng(n)
    x = _inputs(rng, n)
    d0, d1 = hb.hb_share_f32(torch.from_numpy(x).to(DEV), 77 + n)
    e0, e1 = oracle.share_f32(x, 77 + n)
    assert np.array_equal(d0.cpu().numpy(), e0) and np.array_equal(d1.cpu().numpy(), e1)
    y = hb.hb_reveal_f32(d0, d1).cpu().numpy()
    assert np.array_equal(_bits(y), _bits(oracle.reveal_f32(e0, e1)))
    # arbitrary shares (not produced by sharing): the decode of huge ring values
    a = rng.integers(0, 1 << 64, n, dtype=np.uint64).view(np.int64)
    b = rng.integers(0, 1 << 64, n, dtype=np.uint64).view(np.int64)
    y = hb.hb_reveal_f32(torch.from_numpy(a).to(DEV), torch.from_numpy(b).to(DEV)).cpu().numpy()
    assert np.array_equal(_bits(y), _bits(oracle.reveal_f32(a, b)))


@pytest.mark.parametrize("k,m", [(12, 20), (8, 14), (0, 18), (0, 22), (8, 12), (6, 16), (16, 32), (0, 32), (7, 16),
                                 (5, 6), (5, 7), (5, 8), (0, 33), (10, 50), (0, 64), (1, 64)])
def test_simulator_kernel_matches_oracle(k, m):
    w = m - k
    L = min(64 // w, 32)
    rng = np.random.default_rng(k * 64 + m)
    for n in sorted({1, 2, L, 64 * L - 1, 64 * L, 64 * L + 1, 5 * 64 * L + 3, 30001}):
        x = _inputs(rng, n)
        y = hb.hb_sim_relu_f32(torch.from_numpy(x).to(DEV), k, m, SEED, 4242 + n).cpu().numpy()
        e = oracle.sim_relu_f32(x, k, m, SEED, 4242 + n)
        assert np.array_equal(_bits(y), _bits(e)), (k, m, n)


def test_simulator_kernel_at_size_matches_oracle_and_composition_and_in_place():
    """2^23 + 5 floats: every output against the oracle's share -> protocol -> reveal chain, and against the
    library's own three-call composition."""
    n = (1 << 23) + 5
    g = torch.Generator(device=DEV)
    g.manual_seed(3)
    x = torch.randn(n, generator=g, device=DEV, dtype=torch.float32) * 2
    xh = x.cpu().numpy()
    for (k, m) in [(12, 20), (0, 20), (8, 18), (0, 64), (9, 12), (20, 21), (2, 40)]:
        s0, s1 = hb.hb_share_f32(x, 555)
        r0, r1, _ = hb.hb_relu(s0, s1, k, m, SEED)
        ref = hb.hb_reveal_f32(r0, r1)
        y = hb.hb_sim_relu_f32(x, k, m, SEED, 555)
        assert torch.equal(y.view(torch.int32), ref.view(torch.int32))
        e = oracle.sim_relu_f32(xh, k, m, SEED, 555, threads=THREADS)
        assert np.array_equal(_bits(y.cpu().numpy()), _bits(e)), (k, m)
    # full-ring reference through the composable pieces: exactly ReLU of the quantised input
    s0, s1 = hb.hb_share_f32(x, 555)
    r0, r1, _ = hb.hb_relu(s0, s1, 0, 64, SEED)
    exact = hb.hb_reveal_f32(r0, r1)
    q = torch.round(x.double() * 65536.0) / 65536.0
    assert torch.equal(exact, torch.clamp(q, min=0).float())
    z = x.clone()
    hb.hb_sim_relu_f32(z, 12, 20, SEED, 555, out=z)
    assert torch.equal(z.view(torch.int32), hb.hb_sim_relu_f32(x, 12, 20, SEED, 555).view(torch.int32))


def test_float_boundary_errors():
    x = torch.zeros(1001, dtype=torch.float32, device=DEV)
    with pytest.raises(hb.HbError) as e:
        hb.hb_sim_relu_f32(x, 0, 65, SEED, 1)
    assert e.value.status == hb.HB_EINVAL
    with pytest.raises(hb.HbError) as e:
        hb.hb_sim_relu_f32(x[1:], 12, 20, SEED, 1)           # 4-byte aligned only
    assert e.value.status == hb.HB_EALIGN
    with pytest.raises(hb.HbError) as e:
        hb.hb_sim_relu_f32(x, 20, 12, SEED, 1)
    assert e.value.status == hb.HB_EINVAL
    s0, s1 = hb.hb_share_f32(x[1:], 9)                        # the stand-alone kernels take any float alignment
    assert torch.equal(s0 + s1, torch.zeros(1000, dtype=torch.int64, device=DEV))
    assert hb.raw("hb_share_f32", None, 5, 1, s0.data_ptr(), s1.data_ptr(), None) == hb.HB_EINVAL
    assert hb.raw("hb_reveal_f32", s0.data_ptr(), s1.data_ptr(), 5, None, None) == hb.HB_EINVAL
    torch.cuda.synchronize()
