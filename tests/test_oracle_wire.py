"""Pins of the oracle's per-party wire transcript (no GPU).

Each party's wire holds the masked values it sends for every opening.  XORing (adding) the two wires gives
the opened values d, e, z, eps, delta; removing the dealer's masks from them must give what the circuit is
supposed to be operating on at that point, which has a definition that does not involve the protocol at all:
after r prefix rounds, P_r[i] says "bits i-2^r+1 .. i all propagate" and G_r[i] says "adding those bits of
u0 and u1 carries out" (Kogge-Stone; Sec. 2.2 "adder circuit").  These are computed here by brute force with
plain integer arithmetic.  The dealer words are read through the pinned generator (oracle.sm) at the indices
the protocol text assigns.  The byte count of the wire is checked against the closed-form opened-bit count
(Sec. 2.3 / Sec. 4.2 accounting).
"""
import numpy as np
import pytest

import oracle

M64 = (1 << 64) - 1


def _shape(k, m, variant=0):
    w = m - k
    R = 0 if w == 1 else (w - 1).bit_length()
    L = min(64 // w, 32)
    return w, R, L, (5 + 8 * R + 1) if variant else (5 * (1 + 2 * R) + 1)


def _dealer_word(variant, R, gate, slot):
    """Index, inside a group's dealer words, of slot (0: a_0, 1: a_1, 2: b_0, 3: b_1, 4: c_0) of a gate
    (0: gate 0; ("T", r) / ("P", r): the G-update / P-update of round r), written out from the protocol text.
    Shared-mask layout: gate 0 owns words 0..4; round r owns 5 + 8r .. 5 + 8r + 7 =
    a_0 a_1 | b_0 b_1 c_0 (G-update) | b_0 b_1 c_0 (P-update)."""
    if gate == 0:
        return slot
    kind, r = gate
    if not variant:
        return 5 * ((1 if kind == "T" else 2) + 2 * r) + slot
    base = 5 + 8 * r
    if slot < 2:
        return base + slot
    return base + (2 if kind == "T" else 5) + (slot - 2)


def _window_generate(u0, u1, lo, hi):
    """carry out of adding bits lo..hi (inclusive) of u0 and u1 with no carry in; bits below 0 do not exist"""
    lo = max(lo, 0)
    width = hi - lo + 1
    a = (u0 >> lo) & ((1 << width) - 1)
    b = (u1 >> lo) & ((1 << width) - 1)
    return ((a + b) >> width) & 1


def _window_propagate(u0, u1, lo, hi):
    if lo < 0:
        return 0                      # zeros are shifted in: a window reaching below bit 0 does not propagate
    p = u0 ^ u1
    width = hi - lo + 1
    return 1 if ((p >> lo) & ((1 << width) - 1)) == (1 << width) - 1 else 0


@pytest.mark.parametrize("variant", [0, 1])
@pytest.mark.parametrize("k,m", [(12, 20), (0, 64), (8, 14), (8, 18), (3, 4), (0, 2), (5, 12), (20, 53), (8, 12), (0, 33)])
def test_openings_unmask_to_kogge_stone_state(k, m, variant):
    w, R, L, Wg = _shape(k, m, variant)
    per_round = 3 if variant else 4
    rng = np.random.default_rng(k * 64 + m)
    n = 2 * L + max(1, L // 2)
    s0 = rng.integers(0, 1 << 64, n, dtype=np.uint64).view(np.int64)
    s1 = rng.integers(0, 1 << 64, n, dtype=np.uint64).view(np.int64)
    seed = 0xABCDEF + m
    w0, w1 = oracle.relu_wire(s0, s1, k, m, seed, variant)
    w0 = [int(v) for v in w0]
    w1 = [int(v) for v in w1]
    G = (n + L - 1) // L
    assert len(w0) == 2 * G + per_round * G * R + (n + 63) // 64 + 2 * n == oracle.wire_words(n, k, m, variant)
    seedB, seedA = oracle.sm(seed, 0), oracle.sm(seed, 1)
    mask = (1 << w) - 1
    d0, d1, _ = oracle.drelu(s0, s1, k, m, seed, variant=variant)
    for i in range(n):
        g, j = divmod(i, L)
        x0, x1 = int(s0[i]) & M64, int(s1[i]) & M64
        u0, u1 = (x0 >> k) & mask, (x1 >> k) & mask

        def dealer(gate, slot):
            return (oracle.sm(seedB, g * Wg + _dealer_word(variant, R, gate, slot)) >> (j * w)) & mask

        def opened(section_off, per_group, idx):
            pos = section_off + per_group * g + idx
            return ((w0[pos] ^ w1[pos]) >> (j * w)) & mask

        # gate 0: operands are the two slices themselves
        assert opened(0, 2, 0) ^ dealer(0, 0) ^ dealer(0, 1) == u0
        assert opened(0, 2, 1) ^ dealer(0, 2) ^ dealer(0, 3) == u1
        for r in range(R):
            s = 1 << r
            off = 2 * G + per_round * G * r
            P = sum(_window_propagate(u0, u1, b - s + 1, b) << b for b in range(w))
            Gn = sum(_window_generate(u0, u1, b - s + 1, b) << b for b in range(w))
            qT, qP = ("T", r), ("P", r)
            if variant:     # P ^ a travels once and serves both gates
                assert opened(off, 3, 0) ^ dealer(qT, 0) ^ dealer(qT, 1) == P, (i, r)
                assert dealer(qP, 0) == dealer(qT, 0) and dealer(qP, 1) == dealer(qT, 1)
                assert opened(off, 3, 1) ^ dealer(qT, 2) ^ dealer(qT, 3) == (Gn << s) & mask, (i, r)
                assert opened(off, 3, 2) ^ dealer(qP, 2) ^ dealer(qP, 3) == (P << s) & mask, (i, r)
            else:
                assert opened(off, 4, 0) ^ dealer(qT, 0) ^ dealer(qT, 1) == P, (i, r)
                assert opened(off, 4, 1) ^ dealer(qT, 2) ^ dealer(qT, 3) == (Gn << s) & mask, (i, r)
                assert opened(off, 4, 2) ^ dealer(qP, 0) ^ dealer(qP, 1) == P, (i, r)
                assert opened(off, 4, 3) ^ dealer(qP, 2) ^ dealer(qP, 3) == (P << s) & mask, (i, r)
        # B2A: the opened bit is the sign masked by the dealer's bit
        off_b = 2 * G + per_round * G * R
        z = ((w0[off_b + i // 64] ^ w1[off_b + i // 64]) >> (i % 64)) & 1
        wb = oracle.sm(seedB, g * Wg + Wg - 1)
        rbit = ((wb >> (2 * j)) ^ (wb >> (2 * j + 1))) & 1
        sign = ((u0 + u1) >> (w - 1)) & 1
        assert z ^ rbit == sign
        # multiply: eps = x - a, delta = DReLU - b
        off_m = off_b + (n + 63) // 64
        eps = (w0[off_m + 2 * i] + w1[off_m + 2 * i]) & M64
        dlt = (w0[off_m + 2 * i + 1] + w1[off_m + 2 * i + 1]) & M64
        a = (oracle.sm(seedA, 6 * i + 1) + oracle.sm(seedA, 6 * i + 2)) & M64
        b = (oracle.sm(seedA, 6 * i + 3) + oracle.sm(seedA, 6 * i + 4)) & M64
        assert (eps + a) & M64 == (x0 + x1) & M64
        assert (dlt + b) & M64 == (int(d0[i]) + int(d1[i])) & M64 == 1 - sign
    # bits that belong to no element are zero (dead top bits of a word, fields past n in the last group)
    used = n - (G - 1) * L
    live_last = (1 << (used * w)) - 1
    for pos in [2 * (G - 1), 2 * (G - 1) + 1] + [2 * G + per_round * G * r + per_round * (G - 1) + t
                                                for r in range(R) for t in range(per_round)]:
        assert w0[pos] & ~live_last & M64 == 0 and w1[pos] & ~live_last & M64 == 0
    if n % 64:
        tail = off_b + (n + 63) // 64 - 1
        assert w0[tail] >> (n % 64) == 0 and w1[tail] >> (n % 64) == 0


def test_wire_size_is_the_opened_bit_count():
    """When fields fill the words exactly (w * L = 64) and n is a multiple of 64, every wire bit is an opened bit."""
    for (k, m) in [(12, 20), (8, 12), (0, 16), (4, 36), (0, 64), (9, 11)]:
        for n in (64, 640, 4096):
            assert 64 * oracle.wire_words(n, k, m) == oracle.opened_bits(True, k, m, n)
            # one mask of P per round: three words per round instead of four, 3w opened bits instead of 4w
            assert 64 * oracle.wire_words(n, k, m, 1) == oracle.opened_bits(True, k, m, n, variant=1)
    # otherwise the only excess is padding: dead top bits of group words, the ragged last group, the last B2A word
    for (k, m, n) in [(8, 14, 1000), (8, 18, 1000), (12, 20, 1001), (0, 33, 77), (5, 6, 64), (5, 6, 100)]:
        w, R, L, _ = _shape(k, m)
        G = (n + L - 1) // L
        pad = (64 * G - w * n) * (2 + 4 * R) + (64 * ((n + 63) // 64) - n)
        assert 64 * oracle.wire_words(n, k, m) == oracle.opened_bits(True, k, m, n) + pad


def test_wire_is_masked():
    """A party's wire alone looks uniform whatever the inputs are (every opening is masked by dealer material)."""
    rng = np.random.default_rng(8)
    n = 4096
    for inputs in ("zeros", "random"):
        if inputs == "zeros":
            s0 = np.zeros(n, dtype=np.int64)
            s1 = np.zeros(n, dtype=np.int64)
        else:
            s0 = rng.integers(0, 1 << 64, n, dtype=np.uint64).view(np.int64)
            s1 = rng.integers(0, 1 << 64, n, dtype=np.uint64).view(np.int64)
        for wire in oracle.relu_wire(s0, s1, 12, 20, 77):
            density = np.unpackbits(wire.view(np.uint8)).mean()
            assert abs(density - 0.5) < 0.01
