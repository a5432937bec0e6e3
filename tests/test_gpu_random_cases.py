"""Seeded random sweep of the fused entry points against the oracle: random (k, m), sizes around the tile and block
boundaries of that width, random seeds, aligned / 8-byte-aligned buffers, separate or in-place outputs, both dealer
layouts, two-party and multi-party calls.  Everything is integer: the comparison is exact."""
import numpy as np
import pytest
import torch

import oracle
from paper_2309_04875_amd import hb

pytestmark = pytest.mark.gpu

DEV = "cuda"


def _shares(rng, n, parties=2):
    return [rng.integers(0, 1 << 64, n, dtype=np.uint64).view(np.int64) for _ in range(parties)]


def _sizes(rng, w):
    L = min(64 // w, 32)
    tile = (32 if L > 16 else 64) * L                  # elements per wavefront of the tile kernels
    block = 4 * tile
    near = [1, L, tile - 1, tile, tile + 1, block - 1, block, block + 1, 3 * block + tile + 1]
    return int(rng.choice(near)) if rng.random() < 0.6 else int(rng.integers(1, 4 * block))


@pytest.mark.parametrize("chunk", range(8))
def test_random_two_party_cases(chunk):
    rng = np.random.default_rng(1000 + chunk)
    for case in range(40):
        w = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 12, 15, 16, 17, 21, 31, 32, 33, 40, 63, 64]))
        k = int(rng.integers(0, 64 - w + 1))
        m = k + w
        n = _sizes(rng, w)
        seed = int(rng.integers(0, 1 << 63))
        off = int(rng.integers(0, 2))                  # 1: buffers start 8 bytes past a 16-byte boundary
        layout = int(rng.integers(0, 2))
        op = str(rng.choice(["relu", "drelu"]))
        in_place = bool(rng.integers(0, 2))
        s0, s1 = _shares(rng, n)
        what = oracle.WHAT_RELU if op == "relu" else oracle.WHAT_DRELU
        e0, e1 = oracle.evaluate(s0, s1, k, m, seed, what, variant=layout)
        buf0 = torch.empty(n + off, dtype=torch.int64, device=DEV)
        buf1 = torch.empty(n + off, dtype=torch.int64, device=DEV)
        d0, d1 = buf0[off:], buf1[off:]
        d0.copy_(torch.from_numpy(s0))
        d1.copy_(torch.from_numpy(s1))
        if in_place:
            o0, o1 = d0, d1
        else:
            o0 = torch.empty(n + off, dtype=torch.int64, device=DEV)[off:]
            o1 = torch.empty(n + off, dtype=torch.int64, device=DEV)[off:]
        f = hb.hb_relu_ex if op == "relu" else hb.hb_drelu_ex
        f(d0, d1, k, m, seed, layout, o0, o1)
        tag = (chunk, case, op, k, m, n, off, layout, in_place)
        assert np.array_equal(o0.cpu().numpy(), e0), tag
        assert np.array_equal(o1.cpu().numpy(), e1), tag


@pytest.mark.parametrize("parties", [3, 4])
def test_random_multi_party_cases(parties):
    rng = np.random.default_rng(2000 + parties)
    for case in range(30):
        w = int(rng.choice([1, 2, 3, 4, 5, 6, 8, 10, 16, 21, 32, 33, 64]))
        k = int(rng.integers(0, 64 - w + 1))
        m = k + w
        L = min(64 // w, 64 // parties)
        n = int(rng.choice([1, L, 64 * L - 1, 64 * L, 64 * L + 1, 256 * L + 3, int(rng.integers(1, 600 * L))]))
        seed = int(rng.integers(0, 1 << 63))
        off = int(rng.integers(0, 2))
        relu = bool(rng.integers(0, 2))
        sh = _shares(rng, n, parties)
        exp, _ = (oracle.mp_relu if relu else oracle.mp_drelu)(sh, k, m, seed)
        dev = []
        for s in sh:
            b = torch.empty(n + off, dtype=torch.int64, device=DEV)[off:]
            b.copy_(torch.from_numpy(s))
            dev.append(b)
        outs = [torch.empty(n + off, dtype=torch.int64, device=DEV)[off:] for _ in range(parties)]
        (hb.hb_relu_mp if relu else hb.hb_drelu_mp)(dev, k, m, seed, outs)
        for q in range(parties):
            assert np.array_equal(outs[q].cpu().numpy(), exp[q]), (parties, case, relu, k, m, n, off, q)
