"""Second reading of the dealer layout, bit by bit, in pure Python (no GPU).

The paper does not fix where a gate's triple bits or the B2A bit sit inside the dealer streams; that
layout is this project's protocol text.  The reconstructed values are pinned elsewhere; the VALUES OF THE
SHARES are "parity unpinned".  This file does not pin them either: it guards against a slip between the
protocol text and the oracle by evaluating a few elements a different way -- one wire (bit) at a time,
addressing every dealer bit by its absolute position in its 64-bit word -- and comparing share by share.
"""
import numpy as np
import pytest

import oracle

M64 = (1 << 64) - 1
GAMMA = 0x9E3779B97F4A7C15


def _mix(z):
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
    return z ^ (z >> 31)


def _stream(seed, j):
    return _mix((seed + (j + 1) * GAMMA) & M64)


def _bit(word, pos):
    return (word >> pos) & 1


def _group_word_names(R, variant):
    """The dealer words of one group, in stream order, as (gate, slot) names; slots 0..4 = a0 a1 b0 b1 c0."""
    names = [(0, s) for s in range(5)]
    for r in range(R):
        g_gate, p_gate = 1 + 2 * r, 2 + 2 * r
        if variant == 0:        # five words for every gate
            names += [(g_gate, s) for s in range(5)] + [(p_gate, s) for s in range(5)]
        else:                   # one mask of P for the round, then (b0 b1 c0) of each gate
            names += [("mask", r, 0), ("mask", r, 1)]
            names += [(g_gate, s) for s in (2, 3, 4)] + [(p_gate, s) for s in (2, 3, 4)]
    names.append("b2a")
    return names


def _element_bitwise(i, x0, x1, k, m, seed, what, variant=0):
    w = m - k
    R = 0 if w == 1 else (w - 1).bit_length()
    L = min(64 // w, 32)
    names = _group_word_names(R, variant)
    words_per_group = len(names)
    seedB, seedA = _stream(seed, 0), _stream(seed, 1)
    g, lane = divmod(i, L)

    def dealer_bit(gate, slot, b):          # bit b of this element's field in that gate's word
        name = (gate, slot)
        if variant == 1 and gate > 0 and slot < 2:
            name = ("mask", (gate - 1) // 2, slot)
        return _bit(_stream(seedB, g * words_per_group + names.index(name)), lane * w + b)

    def and_wire(gate, b, U, V):            # U, V: (party0 bit, party1 bit) on wire b
        a0, a1, b0, b1, c0 = [dealer_bit(gate, s, b) for s in range(5)]
        c1 = ((a0 ^ a1) & (b0 ^ b1)) ^ c0
        d = U[0] ^ U[1] ^ a0 ^ a1
        e = V[0] ^ V[1] ^ b0 ^ b1
        return (c0 ^ (d & b0) ^ (e & a0) ^ (d & e), c1 ^ (d & b1) ^ (e & a1))

    x0 &= M64
    x1 &= M64
    u0 = [(x0 >> (k + b)) & 1 for b in range(w)]
    u1 = [(x1 >> (k + b)) & 1 for b in range(w)]
    X = [(u0[b], 0) for b in range(w)]
    Y = [(0, u1[b]) for b in range(w)]
    P = [(X[b][0] ^ Y[b][0], X[b][1] ^ Y[b][1]) for b in range(w)]
    S = list(P)
    G = [and_wire(0, b, X[b], Y[b]) for b in range(w)]
    zero = (0, 0)
    for r in range(R):
        s = 1 << r
        Gs = [G[b - s] if b >= s else zero for b in range(w)]
        Ps = [P[b - s] if b >= s else zero for b in range(w)]
        T = [and_wire(1 + 2 * r, b, P[b], Gs[b]) for b in range(w)]
        Pn = [and_wire(2 + 2 * r, b, P[b], Ps[b]) for b in range(w)]
        G = [(G[b][0] ^ T[b][0], G[b][1] ^ T[b][1]) for b in range(w)]
        P = Pn
    carry_in = G[w - 2] if w >= 2 else zero
    sign = (S[w - 1][0] ^ carry_in[0], S[w - 1][1] ^ carry_in[1])
    if what == "sum":       # XOR shares of every sum bit: propagate XOR carry-in
        cin = [zero] + G[:w - 1]
        return tuple(sum((S[b][p] ^ cin[b][p]) << b for b in range(w)) for p in (0, 1))

    wb = _stream(seedB, g * words_per_group + names.index("b2a"))
    rho = (_bit(wb, 2 * lane), _bit(wb, 2 * lane + 1))
    z = sign[0] ^ sign[1] ^ rho[0] ^ rho[1]
    rA0 = _stream(seedA, 6 * i)
    rA1 = ((rho[0] ^ rho[1]) - rA0) & M64
    beta0 = (rA0 + z - 2 * z * rA0) & M64
    beta1 = (rA1 - 2 * z * rA1) & M64
    D = ((1 - beta0) & M64, (-beta1) & M64)
    if what == "drelu":
        return D
    a0, a1, b0, b1, c0 = [_stream(seedA, 6 * i + t) for t in range(1, 6)]
    c1 = ((a0 + a1) * (b0 + b1) - c0) & M64
    eps = (x0 - a0 + x1 - a1) & M64
    dlt = (D[0] - b0 + D[1] - b1) & M64
    return ((c0 + eps * b0 + dlt * a0 + eps * dlt) & M64, (c1 + eps * b1 + dlt * a1) & M64)


@pytest.mark.parametrize("variant", [0, 1])
@pytest.mark.parametrize("k,m", [(12, 20), (0, 64), (8, 14), (8, 18), (3, 4), (0, 2), (5, 8), (20, 53), (8, 12), (0, 33), (7, 39)])
def test_shares_match_bitwise_reading(k, m, variant):
    rng = np.random.default_rng(k * 64 + m)
    w = m - k
    L = min(64 // w, 32)
    n = 3 * L + 2
    s0 = rng.integers(0, 1 << 64, n, dtype=np.uint64).view(np.int64)
    s1 = rng.integers(0, 1 << 64, n, dtype=np.uint64).view(np.int64)
    seed = 0xC0FFEE + m
    d0, d1, _ = oracle.drelu(s0, s1, k, m, seed, variant=variant)
    r0, r1, _ = oracle.relu(s0, s1, k, m, seed, variant=variant)
    b0, b1 = oracle.evaluate(s0, s1, k, m, seed, oracle.WHAT_SUM, variant=variant)
    for i in range(n):
        D = _element_bitwise(i, int(s0[i]), int(s1[i]), k, m, seed, "drelu", variant)
        Rl = _element_bitwise(i, int(s0[i]), int(s1[i]), k, m, seed, "relu", variant)
        B = _element_bitwise(i, int(s0[i]), int(s1[i]), k, m, seed, "sum", variant)
        assert (int(b0[i]) & M64, int(b1[i]) & M64) == B, (i, k, m)
        assert (int(d0[i]) & M64, int(d1[i]) & M64) == D, (i, k, m)
        assert (int(r0[i]) & M64, int(r1[i]) & M64) == Rl, (i, k, m)
