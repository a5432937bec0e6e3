"""Nothing outside [0, n) of any buffer is written: inputs and outputs sit inside larger allocations whose
surroundings hold a sentinel, sizes straddle the tile and block boundaries of each width (the bounds-check-free
body of the tile kernels runs on every wave-tile but a tensor's last), and after each call the sentinels and the
inputs are compared bit for bit."""
import numpy as np
import pytest
import torch

from paper_2309_04875_amd import hb

pytestmark = pytest.mark.gpu

DEV = "cuda"
PAD = 4096                      # elements of padding on each side
SENTINEL = -0x0123456789ABCDEF


def _framed(n, off, fill=None):
    """A view of n elements at offset PAD + off inside a sentinel-filled allocation."""
    whole = torch.full((n + 2 * PAD + 2,), SENTINEL, dtype=torch.int64, device=DEV)
    view = whole[PAD + off:PAD + off + n]
    if fill is not None:
        view.copy_(fill)
    return whole, view


def _intact(whole, n, off):
    lo, hi = PAD + off, PAD + off + n
    return bool((whole[:lo] == SENTINEL).all()) and bool((whole[hi:] == SENTINEL).all())


def _sizes(w, parties=2):
    L = min(64 // w, 32 if parties == 2 else 64 // parties)
    tile = (32 if (parties == 2 and L > 16) else 64) * L
    block = 4 * tile
    return sorted({1, L - 1 or 1, L, L + 1, tile - 1, tile, tile + 1, block - 1, block, block + 1, 2 * block + tile + 3})


@pytest.mark.parametrize("w", [1, 2, 3, 4, 6, 8, 10, 16, 21, 32, 33, 64])
def test_two_party_calls_stay_inside_their_buffers(w):
    g = torch.Generator(device=DEV)
    g.manual_seed(w)
    k = (64 - w) // 2
    for n in _sizes(w):
        for off in (0, 1):
            data = [torch.randint(-2**62, 2**62, (n,), generator=g, device=DEV, dtype=torch.int64) for _ in range(2)]
            w0, s0 = _framed(n, off, data[0])
            w1, s1 = _framed(n, off, data[1])
            for call in (hb.hb_relu, hb.hb_drelu, hb.hb_sign_shares):
                wo0, o0 = _framed(n, off)
                wo1, o1 = _framed(n, off)
                call(s0, s1, k, k + w, 99, o0, o1)
                torch.cuda.synchronize()
                tag = (call.__name__, w, n, off)
                assert _intact(wo0, n, off) and _intact(wo1, n, off), tag
                assert _intact(w0, n, off) and _intact(w1, n, off), tag
                assert torch.equal(s0, data[0]) and torch.equal(s1, data[1]), tag
                assert not bool((o0 == SENTINEL).all()) or n < 4, tag       # the outputs were written
            wo, o = _framed(n, off)
            hb.hb_open(s0, s1, False, out=o)
            torch.cuda.synchronize()
            assert _intact(wo, n, off) and torch.equal(o, data[0] + data[1]), ("open", w, n, off)


def test_batched_and_multi_party_calls_stay_inside_their_buffers():
    g = torch.Generator(device=DEV)
    g.manual_seed(7)
    items, frames = [], []
    for t, (w, n) in enumerate([(8, 511), (8, 512), (8, 513), (8, 2048), (6, 641), (6, 2559), (2, 1023), (10, 385),
                                (8, 1), (64, 300), (8, 4099)]):
        off = t % 2
        bufs = []
        for j in range(4):
            fill = torch.randint(-2**62, 2**62, (n,), generator=g, device=DEV, dtype=torch.int64) if j < 2 else None
            bufs.append(_framed(n, off, fill))
        frames.append((n, off, bufs))
        k = min(12, 64 - w)
        items.append((bufs[0][1], bufs[1][1], bufs[2][1], bufs[3][1], k, k + w, 1000 + t))
    for call in (hb.hb_relu_batch, hb.hb_drelu_batch):
        call(items)
        torch.cuda.synchronize()
        for (n, off, bufs) in frames:
            assert all(_intact(whole, n, off) for (whole, _) in bufs), (call.__name__, n, off)
    for parties in (3, 4):
        for w in (3, 8, 16, 40):
            for n in _sizes(w, parties)[-5:]:
                off = n % 2
                ins = [_framed(n, off, torch.randint(-2**62, 2**62, (n,), generator=g, device=DEV, dtype=torch.int64))
                       for _ in range(parties)]
                outs = [_framed(n, off) for _ in range(parties)]
                hb.hb_relu_mp([v for (_, v) in ins], 5, 5 + w, 77, [v for (_, v) in outs])
                torch.cuda.synchronize()
                assert all(_intact(whole, n, off) for (whole, _) in ins + outs), (parties, w, n, off)
