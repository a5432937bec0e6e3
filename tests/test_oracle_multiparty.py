"""Pins of the p-party oracle (oracle/hb_ref_mp.c), no GPU.

With p = 2 it must be the two-party oracle share for share.  For p > 2 the reconstructed quantities are
pinned by closed forms (plain integer sums of the slices), exactness on the full ring, brute force over
every share triple of a small ring, and a bit-by-bit second reading of the dealer layout with the adder
tree written out by hand.  The values of individual output shares for p > 2 are "parity unpinned".
"""
import numpy as np
import pytest

import oracle

SEED = 0x2309048750000003
M64 = (1 << 64) - 1
GAMMA = 0x9E3779B97F4A7C15


def _rand(rng, p, n):
    return [rng.integers(0, 1 << 64, n, dtype=np.uint64).view(np.int64) for _ in range(p)]


def _u(a):
    return a.view(np.uint64)


def _slices_sum(shares, k, w):
    mask = np.uint64(M64 if w == 64 else (1 << w) - 1)
    tot = np.zeros(shares[0].size, dtype=np.uint64)
    for s in shares:
        tot = tot + ((_u(s) >> np.uint64(k)) & mask)          # wraps mod 2^64, 2^w divides 2^64
    return tot & mask


def _shares_of(x, p, rng):
    sh = [rng.integers(0, 1 << 64, x.size, dtype=np.uint64) for _ in range(p - 1)]
    last = x.view(np.uint64).copy()
    for s in sh:
        last = last - s
    return [s.view(np.int64) for s in sh] + [last.view(np.int64)]


# ---- p = 2 is the two-party protocol ---------------------------------------------------------------------------

@pytest.mark.parametrize("k,m", [(12, 20), (0, 64), (8, 14), (0, 1), (63, 64), (5, 38), (3, 4), (0, 2), (7, 39), (8, 18)])
def test_two_parties_reproduce_the_two_party_oracle(k, m):
    rng = np.random.default_rng(k * 64 + m)
    w = m - k
    L = min(64 // w, 32)
    s = _rand(rng, 2, 5 * L + 3)
    for what in (oracle.WHAT_DRELU, oracle.WHAT_RELU, oracle.WHAT_SUM, oracle.WHAT_SIGN, oracle.WHAT_SLICE):
        a = oracle.mp_evaluate(s, k, m, SEED, what)
        b = oracle.evaluate(s[0], s[1], k, m, SEED, what)
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]), what
    assert oracle.mp_opened_bits(True, 2, k, m, 7) == oracle.opened_bits(True, k, m, 7)
    assert oracle.mp_opened_bits(False, 2, k, m, 7) == oracle.opened_bits(False, k, m, 7)


def test_two_parties_small_ring_reproduces_too():
    v = np.arange(256, dtype=np.int64)
    s0, s1 = [a.reshape(-1) for a in np.meshgrid(v, v, indexing="ij")]
    for (k, m) in [(0, 8), (2, 5), (1, 8), (3, 4)]:
        a = oracle.mp_evaluate([s0, s1], k, m, SEED, oracle.WHAT_RELU, ring_bits=8)
        b = oracle.evaluate(s0, s1, k, m, SEED, oracle.WHAT_RELU, ring_bits=8)
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


# ---- the adder tree ------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("p", [3, 4, 5, 8])
@pytest.mark.parametrize("w", [1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 12, 16, 17, 21, 22, 31, 32, 33, 48, 63, 64])
def test_adder_tree_reconstructs_plain_sum(p, w):
    """XOR of the p sum shares == (sum of the p slices) mod 2^w in ALL w bits; sign shares are its top bit."""
    rng = np.random.default_rng(100 * p + w)
    L = min(64 // w, 64 // p)
    n = 11 * L + L // 2 + 1
    i64 = np.iinfo(np.int64)
    for k in sorted({0, 64 - w, (64 - w) // 2}):
        s = _rand(rng, p, n)
        for q in range(p):
            s[q][:3] = [0, -1, i64.min] if q % 2 == 0 else [-1, i64.max, 1]
        b = oracle.mp_evaluate(s, k, k + w, SEED + w, oracle.WHAT_SUM)
        got = np.zeros(n, dtype=np.uint64)
        for q in range(p):
            got ^= _u(b[q])
        assert np.array_equal(got, _slices_sum(s, k, w)), (p, w, k)
        g = oracle.mp_evaluate(s, k, k + w, SEED + w, oracle.WHAT_SIGN)
        sg = np.zeros(n, dtype=np.uint64)
        for q in range(p):
            assert set(np.unique(g[q])) <= {0, 1}
            sg ^= _u(g[q])
        assert np.array_equal(sg, got >> np.uint64(w - 1))
        u = oracle.mp_evaluate(s, k, k + w, SEED + w, oracle.WHAT_SLICE)
        mask = np.uint64(M64 if w == 64 else (1 << w) - 1)
        for q in range(p):
            assert np.array_equal(_u(u[q]), (_u(s[q]) >> np.uint64(k)) & mask)


@pytest.mark.parametrize("p", [3, 4])
def test_adder_tree_exhaustive_w3(p):
    w = 3
    vals = np.arange(1 << w, dtype=np.int64)
    grids = [a.reshape(-1) for a in np.meshgrid(*([vals] * p), indexing="ij")]
    rng = np.random.default_rng(p)
    s = [(g | (rng.integers(0, 1 << 40, g.size, dtype=np.int64) << w)) << 2 for g in grids]   # junk above, k = 2
    b = oracle.mp_evaluate(s, 2, 2 + w, SEED, oracle.WHAT_SUM)
    got = b[0].copy()
    for q in range(1, p):
        got ^= b[q]
    assert np.array_equal(got, sum(grids) & ((1 << w) - 1))


# ---- exactness and Beaver identities ---------------------------------------------------------------------------------

@pytest.mark.parametrize("p", [3, 4, 7])
def test_full_ring_is_exact(p):
    rng = np.random.default_rng(40 + p)
    i64 = np.iinfo(np.int64)
    x = np.concatenate([
        np.array([0, 1, -1, 2, -2, i64.min, i64.max, i64.min + 1, i64.max - 1, 65536, -65536], dtype=np.int64),
        rng.integers(i64.min, i64.max, 2000, dtype=np.int64),
        np.rint(rng.standard_normal(2000) * 2 * 65536).astype(np.int64),
    ])
    s = _shares_of(x, p, rng)
    d, bits = oracle.mp_drelu(s, 0, 64, SEED)
    assert np.array_equal(sum(d), (x >= 0).astype(np.int64))
    r, rbits = oracle.mp_relu(s, 0, 64, SEED)
    assert np.array_equal(sum(r), np.maximum(x, 0))
    assert rbits - bits == 128 * x.size


@pytest.mark.parametrize("p", [3, 4, 6])
@pytest.mark.parametrize("k,m", [(12, 20), (8, 14), (0, 1), (63, 64), (5, 38), (16, 26), (0, 33)])
def test_beaver_identities_any_slice(p, k, m):
    rng = np.random.default_rng(p * 1000 + k * 64 + m)
    x = np.rint(rng.standard_normal(3000) * 3 * 65536).astype(np.int64)
    x[:3] = [0, -1, 1]
    s = _shares_of(x, p, rng)
    w = m - k
    msb = _slices_sum(s, k, w) >> np.uint64(w - 1)
    expect = 1 - msb.astype(np.int64)
    d, _ = oracle.mp_drelu(s, k, m, SEED)
    assert np.array_equal(sum(d), expect)
    r, _ = oracle.mp_relu(s, k, m, SEED)
    assert np.array_equal(sum(r), x * expect)


def test_window_of_correctness_three_parties():
    """Inside (p-1) 2^k <= |x| and x within the high-cut window the approximate DReLU is right: the dropped low
    carry is at most p - 1 (Sec. 3.1.2's two steps, with the carry bound of p parties)."""
    rng = np.random.default_rng(8)
    p, k, m = 3, 12, 22
    x = rng.integers(-(1 << (m - 1)) + 2 * (1 << k), (1 << (m - 1)), 20000, dtype=np.int64)
    x = x[(x >= 2 * (1 << k)) | (x < 0)]
    s = _shares_of(x, p, rng)
    d, _ = oracle.mp_drelu(s, k, m, SEED)
    assert np.array_equal(sum(d), (x >= 0).astype(np.int64))


def test_brute_force_small_ring_three_parties():
    """Ring Z_2^5, every share triple, every (k, m): what the slices encode and where the result is right."""
    N, p = 5, 3
    v = np.arange(1 << N, dtype=np.int64)
    s = [a.reshape(-1) for a in np.meshgrid(v, v, v, indexing="ij")]
    ring = (1 << N) - 1
    xs = (s[0] + s[1] + s[2]) & ring
    x = np.where(xs >= (1 << (N - 1)), xs - (1 << N), xs)
    checked = 0
    for k in range(N):
        for m in range(k + 1, N + 1):
            w = m - k
            d = oracle.mp_evaluate(s, k, m, SEED, oracle.WHAT_DRELU, ring_bits=N)
            dd = (d[0] + d[1] + d[2]) & ring
            assert set(np.unique(dd)) <= {0, 1}
            r = oracle.mp_evaluate(s, k, m, SEED, oracle.WHAT_RELU, ring_bits=N)
            rr = (r[0] + r[1] + r[2]) & ring
            assert np.array_equal(rr, (xs * dd) & ring)
            low = (1 << k) - 1
            c = ((s[0] & low) + (s[1] & low) + (s[2] & low)) >> k            # dropped low carry, 0 .. p-1
            assert c.max() <= p - 1
            xm = xs & ((1 << m) - 1)
            enc = ((xm >> k) - c) & ((1 << w) - 1)
            assert np.array_equal(dd, 1 - (enc >> (w - 1)))
            half = 1 << (m - 1)
            sure_pos = (x >= (p - 1) * (1 << k)) & (x < half)
            sure_neg = (x >= -half + (p - 1) * (1 << k)) & (x < 0)
            assert (dd[sure_pos] == 1).all() and (dd[sure_neg] == 0).all()
            if (k, m) == (0, N):
                assert np.array_equal(dd, (x >= 0).astype(np.int64))
                assert np.array_equal(rr, np.maximum(x, 0) & ring)
            checked += 1
    assert checked == 15


# ---- counts, host logic ------------------------------------------------------------------------------------------

def test_opened_bits_per_link():
    for p in range(2, 9):
        for w in (1, 4, 8, 10, 64):
            R = 0 if w == 1 else int(np.ceil(np.log2(w)))
            per = (p - 1) * 2 * w * (1 + 2 * R) + 1
            assert oracle.mp_opened_bits(False, p, 0, w, 5) == 5 * per
            assert oracle.mp_opened_bits(True, p, 64 - w, 64, 1) == per + 128
    assert oracle.mp_opened_bits(True, 1, 0, 8, 1) == 0 and oracle.mp_opened_bits(True, 9, 0, 8, 1) == 0
    assert oracle.mp_opened_bits(True, 3, 8, 8, 1) == 0


def test_range_scatter_threads_and_validation():
    rng = np.random.default_rng(5)
    n = 9001
    s = _rand(rng, 3, n)
    a = oracle.mp_evaluate(s, 12, 20, SEED, oracle.WHAT_RELU)
    t = oracle.mp_evaluate(s, 12, 20, SEED, oracle.WHAT_RELU, threads=3)
    assert all(np.array_equal(a[q], t[q]) for q in range(3))
    idx = rng.choice(n, 400, replace=False)
    g = oracle.mp_evaluate_at([x[idx] for x in s], idx.astype(np.uint64), 12, 20, SEED, oracle.WHAT_RELU)
    assert all(np.array_equal(g[q], a[q][idx]) for q in range(3))
    c = oracle.mp_evaluate([x[1000:2000] for x in s], 12, 20, SEED, oracle.WHAT_RELU, first=1000)
    assert all(np.array_equal(c[q], a[q][1000:2000]) for q in range(3))
    z = [np.zeros(4, dtype=np.int64)] * 3
    for (k, m) in [(-1, 4), (4, 4), (0, 65)]:
        with pytest.raises(ValueError):
            oracle.mp_evaluate(z, k, m, SEED, oracle.WHAT_RELU)
    with pytest.raises(ValueError):
        oracle.mp_evaluate([np.zeros(4, dtype=np.int64)], 0, 8, SEED, oracle.WHAT_RELU)        # one party
    with pytest.raises(ValueError):
        oracle.mp_evaluate([np.zeros(4, dtype=np.int64)] * 9, 0, 8, SEED, oracle.WHAT_RELU)    # too many


# ---- second reading of the layout, one wire at a time, trees written out ---------------------------------------

def _mix(z):
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
    return z ^ (z >> 31)


def _stream(seed, j):
    return _mix((seed + (j + 1) * GAMMA) & M64)


def _xor_all(v):
    r = 0
    for t in v:
        r ^= t
    return r


def _element_bitwise(p, i, xs, k, m, seed, what):
    w = m - k
    R = 0 if w == 1 else (w - 1).bit_length()
    L = min(64 // w, 64 // p)
    gates_per_adder = 1 + 2 * R
    words_per_gate = 3 * p - 1
    words_per_group = (p - 1) * gates_per_adder * words_per_gate + 1
    seedB, seedA = _stream(seed, 0), _stream(seed, 1)
    g, lane = divmod(i, L)

    def dealer_bit(adder, gate, slot, b):
        word = g * words_per_group + (adder * gates_per_adder + gate) * words_per_gate + slot
        return (_stream(seedB, word) >> (lane * w + b)) & 1

    def and_wire(adder, gate, b, U, V):            # U, V: tuples of p share bits of wire b
        a = [dealer_bit(adder, gate, q, b) for q in range(p)]
        bb = [dealer_bit(adder, gate, p + q, b) for q in range(p)]
        c = [dealer_bit(adder, gate, 2 * p + q, b) for q in range(p - 1)]
        c.append((_xor_all(a) & _xor_all(bb)) ^ _xor_all(c))
        d = _xor_all(U) ^ _xor_all(a)
        e = _xor_all(V) ^ _xor_all(bb)
        z = [c[q] ^ (d & bb[q]) ^ (e & a[q]) for q in range(p)]
        z[0] ^= d & e
        return tuple(z)

    zero = (0,) * p

    def xor2(A, B):
        return tuple(x ^ y for x, y in zip(A, B))

    def add(adder, X, Y):                           # X, Y: lists over wires of p-tuples
        P = [xor2(X[b], Y[b]) for b in range(w)]
        S = list(P)
        G = [and_wire(adder, 0, b, X[b], Y[b]) for b in range(w)]
        for r in range(R):
            sft = 1 << r
            Gs = [G[b - sft] if b >= sft else zero for b in range(w)]
            Ps = [P[b - sft] if b >= sft else zero for b in range(w)]
            T = [and_wire(adder, 1 + 2 * r, b, P[b], Gs[b]) for b in range(w)]
            Pn = [and_wire(adder, 2 + 2 * r, b, P[b], Ps[b]) for b in range(w)]
            G = [xor2(G[b], T[b]) for b in range(w)]
            P = Pn
        cin = [zero] + G[:w - 1]
        return [xor2(S[b], cin[b]) for b in range(w)]

    xs = [x & M64 for x in xs]
    X = []
    for q in range(p):
        X.append([tuple(((xs[q] >> (k + b)) & 1) if t == q else 0 for t in range(p)) for b in range(w)])
    if p == 3:
        total = add(1, add(0, X[0], X[1]), X[2])
    elif p == 4:
        total = add(2, add(0, X[0], X[1]), add(1, X[2], X[3]))
    elif p == 5:
        total = add(3, add(2, add(0, X[0], X[1]), add(1, X[2], X[3])), X[4])
    else:
        raise AssertionError
    if what == "sum":
        return tuple(sum(total[b][q] << b for b in range(w)) for q in range(p))
    sign = total[w - 1]
    wb = _stream(seedB, g * words_per_group + words_per_group - 1)
    rho = [(wb >> (p * lane + q)) & 1 for q in range(p)]
    z = _xor_all(sign) ^ _xor_all(rho)
    words = 4 * p - 2
    rA = [_stream(seedA, words * i + q) for q in range(p - 1)]
    rA.append((_xor_all(rho) - sum(rA)) & M64)
    D = [((1 if q == 0 else 0) - (rA[q] + (z if q == 0 else 0) - 2 * z * rA[q])) & M64 for q in range(p)]
    if what == "drelu":
        return tuple(D)
    base = words * i + (p - 1)
    a = [_stream(seedA, base + q) for q in range(p)]
    b = [_stream(seedA, base + p + q) for q in range(p)]
    c = [_stream(seedA, base + 2 * p + q) for q in range(p - 1)]
    c.append((sum(a) * sum(b) - sum(c)) & M64)
    eps = (sum(xs) - sum(a)) & M64
    dlt = (sum(D) - sum(b)) & M64
    return tuple((c[q] + eps * b[q] + dlt * a[q] + (eps * dlt if q == 0 else 0)) & M64 for q in range(p))


@pytest.mark.parametrize("p", [3, 4, 5])
@pytest.mark.parametrize("k,m", [(12, 20), (0, 64), (8, 14), (3, 4), (0, 2), (5, 8), (20, 53), (0, 33)])
def test_shares_match_bitwise_reading(p, k, m):
    rng = np.random.default_rng(p * 4096 + k * 64 + m)
    w = m - k
    L = min(64 // w, 64 // p)
    n = 2 * L + 2
    s = _rand(rng, p, n)
    seed = 0xC0FFEE + m
    d = oracle.mp_evaluate(s, k, m, seed, oracle.WHAT_DRELU)
    r = oracle.mp_evaluate(s, k, m, seed, oracle.WHAT_RELU)
    b = oracle.mp_evaluate(s, k, m, seed, oracle.WHAT_SUM)
    for i in range(n):
        xs = [int(a[i]) for a in s]
        assert tuple(int(a[i]) & M64 for a in b) == _element_bitwise(p, i, xs, k, m, seed, "sum"), (i, k, m)
        assert tuple(int(a[i]) & M64 for a in d) == _element_bitwise(p, i, xs, k, m, seed, "drelu"), (i, k, m)
        assert tuple(int(a[i]) & M64 for a in r) == _element_bitwise(p, i, xs, k, m, seed, "relu"), (i, k, m)
