"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU).

Every check here computes its expectation without the oracle: printed values from the paper
(tests/golden/paper_examples.txt), published generator vectors (tests/golden/splitmix64_kat.txt),
plain integer addition, sign tests, exhaustive truth tables and brute force on an 8-bit ring.
"""
import itertools
import os

import numpy as np
import pytest

import oracle
from conftest import GOLDEN

U64 = (1 << 64) - 1
SEED = 0x2309048750000001


def _u64(a):
    return np.asarray(a).astype(np.int64).view(np.uint64)


def _signed(v, bits):
    """Python int / object array: value of the low `bits` bits read as two's complement."""
    v = v & ((1 << bits) - 1)
    return v - (1 << bits) if v >> (bits - 1) else v


def _rand_shares(rng, n):
    return (rng.integers(0, 1 << 64, n, dtype=np.uint64).view(np.int64),
            rng.integers(0, 1 << 64, n, dtype=np.uint64).view(np.int64))


def _slice_np(share, k, w):
    mask = np.uint64(U64 if w == 64 else (1 << w) - 1)
    return (_u64(share) >> np.uint64(k)) & mask


def _sum_mod_2w(u0, u1, w):
    """(u0 + u1) mod 2^w by plain unsigned addition (numpy wraps mod 2^64, then mask)."""
    mask = np.uint64(U64 if w == 64 else (1 << w) - 1)
    return (u0 + u1) & mask


# ----------------------------------------------------------------------------------------------
# dealer generator
# ----------------------------------------------------------------------------------------------

def _read_kat():
    out = []
    with open(os.path.join(GOLDEN, "splitmix64_kat.txt")) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if line:
                seed, vals = line.split(":")
                out.append((int(seed.strip(), 0), [int(v, 0) for v in vals.split()]))
    return out


def test_splitmix64_known_answers():
    kat = _read_kat()
    assert len(kat) == 2
    for seed, vals in kat:
        assert oracle.sm_sequence(seed, len(vals)) == vals           # stepping the generator
        assert [oracle.sm(seed, j) for j in range(len(vals))] == vals  # indexed access


def test_indexed_access_equals_stepping():
    for seed in (0, 1, SEED, U64, 0x8000000000000000):
        seq = oracle.sm_sequence(seed, 300)
        assert [oracle.sm(seed, j) for j in range(300)] == seq


def test_tensor_seed_is_root_stream_from_third_output():
    seq = oracle.sm_sequence(SEED, 12)
    assert [oracle.tensor_seed(SEED, t) for t in range(10)] == seq[2:]


# ----------------------------------------------------------------------------------------------
# values the paper prints
# ----------------------------------------------------------------------------------------------

def test_notation_example_slice(paper_examples):
    p = paper_examples
    s0 = np.array([p["notation_x"]], dtype=np.int64)
    s1 = np.zeros(1, dtype=np.int64)
    u0, u1 = oracle.evaluate(s0, s1, p["notation_lo"], p["notation_hi"], SEED, oracle.WHAT_SLICE)
    assert int(u0[0]) == p["notation_slice"] and int(u1[0]) == 0


@pytest.mark.parametrize("ring_bits", [64, 8])
def test_worked_example(paper_examples, ring_bits):
    p = paper_examples
    k, m = p["example_lo"], p["example_hi"]
    w = m - k
    assert 1 << w == p["example_small_ring"]
    ring = (1 << ring_bits) - 1
    s0 = np.array([p["example_share0"]], dtype=np.int64)
    s1 = np.array([p["example_share1"]], dtype=np.int64)
    assert int(s0[0] + s1[0]) == p["example_x"]
    if ring_bits < 64:  # the same shares written on the small ring
        s0, s1 = s0 & ring, s1 & ring
    u0, u1 = oracle.evaluate(s0, s1, k, m, SEED, oracle.WHAT_SLICE, ring_bits)
    assert int(u0[0]) == p["example_slice0"] % (1 << w)
    assert int(u1[0]) == p["example_slice1"] % (1 << w)
    b0, b1 = oracle.evaluate(s0, s1, k, m, SEED, oracle.WHAT_SUM, ring_bits)
    assert _signed(int(b0[0]) ^ int(b1[0]), w) == p["example_small_secret"]
    d0, d1, _ = oracle.drelu(s0, s1, k, m, SEED, ring_bits)
    assert (int(d0[0]) + int(d1[0])) & ring == p["example_drelu"]
    r0, r1, _ = oracle.relu(s0, s1, k, m, SEED, ring_bits)
    assert (int(r0[0]) + int(r1[0])) & ring == p["example_relu"]


def test_opened_bits_reproduce_paper_breakdown(paper_examples):
    """At w = 64 the per-element openings are 2 units of 64 bits for gate 0 ("Others"), 6 rounds x 2
    gates x 2 units ("Circuit"), B2A and the multiply (2 units).  With B2A sent as a whole 64-bit word, as
    the unpacked baseline does, the shares of the total are the paper's percentages."""
    p = paper_examples
    w = 64
    total_packed = oracle.opened_bits(True, 0, 64, 1)
    drelu_packed = oracle.opened_bits(False, 0, 64, 1)
    mult = total_packed - drelu_packed
    assert mult == 128
    b2a_packed = 1
    circuit_and_others = drelu_packed - b2a_packed
    others = 2 * w
    circuit = circuit_and_others - others
    assert circuit == 6 * 2 * 2 * w
    b2a_unpacked = 64
    total = circuit + others + b2a_unpacked + mult
    assert total == 29 * 64
    assert round(100.0 * circuit / total, 2) == p["comm_circuit_pct"]
    assert round(100.0 * mult / total, 2) == p["comm_mult_pct"]
    assert round(100.0 * b2a_unpacked / total, 2) == p["comm_b2a_pct"]
    assert round(100.0 * others / total, 2) == p["comm_others_pct"]


def test_opened_bits_table_and_scaling():
    # rounds = ceil(log2 w): one opening of 2w bits, then 4w bits per round, 1 bit for B2A, 128 for the multiply
    def expect(w, relu):
        rounds = 0 if w == 1 else int(np.ceil(np.log2(w)))
        return 2 * w + rounds * 4 * w + 1 + (128 if relu else 0)
    for w in range(1, 65):
        for k in (0, 64 - w):
            assert oracle.opened_bits(True, k, k + w, 1) == expect(w, True)
            assert oracle.opened_bits(False, k, k + w, 7) == 7 * expect(w, False)
    printed = {64: 1793, 32: 833, 16: 417, 10: 309, 8: 241, 6: 213, 4: 169}
    for w, bits in printed.items():
        assert oracle.opened_bits(True, 0, w, 1) == bits
    assert oracle.opened_bits(True, 3, 3, 5) == 0 and oracle.opened_bits(True, 0, 65, 5) == 0


def test_reduction_bands_of_the_paper(paper_examples):
    """Sanity band, not an equality: the paper's reductions are end-to-end (linear layers and the parts of ReLU
    that do not shrink included), ours are for the ReLU openings alone, so ours must reach at least the paper's
    lower ends and sit at the paper's upper end for the widths its search keeps.  Kept bits: 64 x (9..13) % = 6..8.
    Rounds of one ReLU: gate 0, ceil(log2 w) prefix rounds, B2A, multiply (the party-wise transcript has one message
    per round); 9 on the full ring."""
    p = paper_examples
    base_bits = 29 * 64
    kept = [w for w in range(1, 65)
            if p["bits_discarded_pct_lo"] <= round(100.0 * (64 - w) / 64.0) <= p["bits_discarded_pct_hi"]]
    assert kept == [6, 7, 8]
    ratios = [base_bits / oracle.opened_bits(True, 12, 12 + w, 1) for w in kept]
    # the multiply (128 bits) does not shrink: the ratio saturates just below the paper's best figure
    assert all(p["bytes_reduction_lo"] < r for r in ratios)
    assert abs(max(ratios) - p["bytes_reduction_hi"]) < 0.1 and max(ratios) <= p["bytes_reduction_hi"]
    # zero-error strategy: 18..22 kept bits, no low cut
    eco = [base_bits / oracle.opened_bits(True, 0, m, 1) for m in range(int(p["eco_kept_bits_lo"]), int(p["eco_kept_bits_hi"]) + 1)]
    assert all(p["bytes_reduction_lo"] < r < p["bytes_reduction_hi"] for r in eco)

    def rounds(w):
        return 1 + (0 if w == 1 else (w - 1).bit_length()) + 2
    assert rounds(64) == 9
    # the paper's least reduction of rounds, 1.12x, is 9 / 8: widths 17..32; 9 / 6 = 1.5 at the kept widths
    assert round(rounds(64) / rounds(32), 2) in (p["rounds_reduction_lo"], round(p["rounds_reduction_lo"] + 0.01, 2))
    assert all(p["rounds_reduction_lo"] <= rounds(64) / rounds(w) <= p["rounds_reduction_hi"] for w in kept + [20, 22, 32])


def test_opened_bits_shared_mask_variant():
    """One mask for P per prefix round: that round opens P ^ a once and two second operands, 3w bits."""
    for w in range(1, 65):
        rounds = 0 if w == 1 else int(np.ceil(np.log2(w)))
        per = 2 * w + 3 * w * rounds + 1
        assert oracle.opened_bits(False, 0, w, 3, variant=1) == 3 * per
        assert oracle.opened_bits(True, 64 - w, 64, 1, variant=1) == per + 128
        saved = oracle.opened_bits(True, 0, w, 1) - oracle.opened_bits(True, 0, w, 1, variant=1)
        assert saved == w * rounds
    # the A2B share of the baseline's 1856 bits falls from 1536 to 1152 + 128 = 1280 (6 rounds of 64 bits saved)
    assert oracle.opened_bits(True, 0, 64, 1, variant=1) == 1793 - 6 * 64
    assert oracle.opened_bits(True, 12, 20, 1, variant=1) == 241 - 24


def test_variants_differ_in_shares_only():
    """The two dealer layouts give different shares of the same reconstructed values (and share gate 0's words)."""
    rng = np.random.default_rng(77)
    s0, s1 = _rand_shares(rng, 4000)
    for (k, m) in [(12, 20), (0, 64), (8, 14), (0, 1)]:
        a0, a1 = oracle.evaluate(s0, s1, k, m, SEED, oracle.WHAT_SUM, variant=0)
        b0, b1 = oracle.evaluate(s0, s1, k, m, SEED, oracle.WHAT_SUM, variant=1)
        assert np.array_equal(a0 ^ a1, b0 ^ b1)
        if m - k > 1:
            assert not np.array_equal(a0, b0)
        r0, r1, _ = oracle.relu(s0, s1, k, m, SEED, variant=0)
        q0, q1, _ = oracle.relu(s0, s1, k, m, SEED, variant=1)
        assert np.array_equal(r0 + r1, q0 + q1)
    with pytest.raises(ValueError):
        oracle.evaluate(s0, s1, 12, 20, SEED, oracle.WHAT_SUM, variant=2)


# ----------------------------------------------------------------------------------------------
# the AND gate and the adder
# ----------------------------------------------------------------------------------------------

def test_and_gate_truth_table():
    for bits in itertools.product((0, 1), repeat=9):
        U0, U1, V0, V1, a0, a1, b0, b1, c0 = bits
        z0, z1 = oracle.and_gate(U0, U1, V0, V1, a0, a1, b0, b1, c0, 1)
        assert z0 ^ z1 == (U0 ^ U1) & (V0 ^ V1), bits


def test_and_gate_words():
    rng = np.random.default_rng(7)
    for _ in range(200):
        v = [int(t) for t in rng.integers(0, 1 << 64, 9, dtype=np.uint64)]
        for mask in (U64, 0xFF, (1 << 37) - 1):
            z0, z1 = oracle.and_gate(*v, mask)
            assert z0 ^ z1 == ((v[0] ^ v[1]) & (v[2] ^ v[3])) & mask
            assert z0 <= mask and z1 <= mask


@pytest.mark.parametrize("variant", [0, 1])
@pytest.mark.parametrize("w", range(1, 65))
def test_adder_reconstructs_plain_sum_every_width(w, variant):
    """XOR of the two sum shares == (u0 + u1) mod 2^w in ALL w bits, for several k and many shares,
    at sizes that cover many dealer groups and a ragged last group."""
    rng = np.random.default_rng(1000 + w)
    L = min(64 // w, 32)
    n = 37 * L + (L // 2) + 1
    for k in sorted({0, (64 - w) // 2, 64 - w}):
        s0, s1 = _rand_shares(rng, n)
        # extremes in front
        s0[:4] = np.array([0, -1, np.iinfo(np.int64).min, np.iinfo(np.int64).max])
        s1[:4] = np.array([-1, -1, np.iinfo(np.int64).min, 1])
        b0, b1 = oracle.evaluate(s0, s1, k, k + w, SEED + w, oracle.WHAT_SUM, variant=variant)
        u0, u1 = _slice_np(s0, k, w), _slice_np(s1, k, w)
        got = _u64(b0) ^ _u64(b1)
        assert np.array_equal(got, _sum_mod_2w(u0, u1, w)), (w, k)
        g0, g1 = oracle.evaluate(s0, s1, k, k + w, SEED + w, oracle.WHAT_SIGN, variant=variant)
        assert np.array_equal(_u64(g0) ^ _u64(g1), got >> np.uint64(w - 1))
        assert set(np.unique(g0)) <= {0, 1} and set(np.unique(g1)) <= {0, 1}


@pytest.mark.parametrize("variant", [0, 1])
@pytest.mark.parametrize("w", range(1, 7))
def test_adder_exhaustive_small_widths(w, variant):
    vals = np.arange(1 << w, dtype=np.int64)
    u0, u1 = [a.reshape(-1) for a in np.meshgrid(vals, vals, indexing="ij")]
    rng = np.random.default_rng(w)
    # random junk above the slice must not matter
    junk0 = rng.integers(0, 1 << 62, u0.size, dtype=np.int64) << w if w < 2 else (rng.integers(0, 1 << 50, u0.size, dtype=np.int64) << w)
    junk1 = rng.integers(0, 1 << 50, u0.size, dtype=np.int64) << w
    for k in (0, 5):
        s0 = ((u0 | junk0) << k) | int(rng.integers(0, 1 << k)) if k else (u0 | junk0)
        s1 = ((u1 | junk1) << k) | int(rng.integers(0, 1 << k)) if k else (u1 | junk1)
        b0, b1 = oracle.evaluate(s0, s1, k, k + w, SEED, oracle.WHAT_SUM, variant=variant)
        assert np.array_equal(b0 ^ b1, (u0 + u1) & ((1 << w) - 1))


# ----------------------------------------------------------------------------------------------
# exactness on the full ring; Beaver identities
# ----------------------------------------------------------------------------------------------

def _shares_of(x, rng):
    s0 = rng.integers(0, 1 << 64, x.size, dtype=np.uint64)
    return s0.view(np.int64), (x.view(np.uint64) - s0).view(np.int64)


@pytest.mark.parametrize("variant", [0, 1])
def test_full_ring_is_exact(variant):
    """(k, m) = (0, 64): DReLU == [x >= 0] and ReLU == max(x, 0) for every x, including the extremes."""
    rng = np.random.default_rng(11)
    i64 = np.iinfo(np.int64)
    x = np.concatenate([
        np.array([0, 1, -1, 2, -2, i64.min, i64.max, i64.min + 1, i64.max - 1, 65536, -65536], dtype=np.int64),
        rng.integers(i64.min, i64.max, 3000, dtype=np.int64),
        np.rint(rng.standard_normal(3000) * 2 * 65536).astype(np.int64),
    ])
    s0, s1 = _shares_of(x, rng)
    d0, d1, bits = oracle.drelu(s0, s1, 0, 64, SEED, variant=variant)
    assert np.array_equal(d0 + d1, (x >= 0).astype(np.int64))
    r0, r1, _ = oracle.relu(s0, s1, 0, 64, SEED, variant=variant)
    assert np.array_equal(r0 + r1, np.maximum(x, 0))
    assert bits == x.size * (oracle.opened_bits(True, 0, 64, 1, variant) - 128)


@pytest.mark.parametrize("k,m", [(0, 64), (12, 20), (8, 16), (0, 1), (63, 64), (5, 38), (8, 14), (16, 26), (0, 33), (31, 64)])
@pytest.mark.parametrize("variant", [0, 1])
def test_beaver_identities_any_slice(k, m, variant):
    """DReLU shares sum to 1 - MSB_w((u0 + u1) mod 2^w) in {0, 1}; ReLU shares sum to x * that, always."""
    rng = np.random.default_rng(k * 100 + m)
    n = 5000
    x = np.rint(rng.standard_normal(n) * 3 * 65536).astype(np.int64)
    x[:3] = [0, -1, 1]
    s0, s1 = _shares_of(x, rng)
    w = m - k
    msb = _sum_mod_2w(_slice_np(s0, k, w), _slice_np(s1, k, w), w) >> np.uint64(w - 1)
    expect_d = (1 - msb.astype(np.int64))
    d0, d1, _ = oracle.drelu(s0, s1, k, m, SEED, variant=variant)
    assert np.array_equal(d0 + d1, expect_d)
    r0, r1, _ = oracle.relu(s0, s1, k, m, SEED, variant=variant)
    assert np.array_equal(r0 + r1, x * expect_d)
    # the DReLU shares inside hb_relu are the ones hb_drelu returns: ReLU opens delta = DReLU - b
    # (checked indirectly: same reconstructed product for every element)


def test_theorem1_high_cut_is_exact_in_range():
    """Dropping bits >= m leaves DReLU unchanged whenever -2^(m-1) <= x < 2^(m-1) (Theorem 1)."""
    rng = np.random.default_rng(21)
    for m in (2, 9, 18, 22, 40, 63):
        lo, hi = -(1 << (m - 1)), (1 << (m - 1))
        x = rng.integers(lo, hi, 4000, dtype=np.int64)
        x[:4] = [lo, hi - 1, 0, -1]
        s0, s1 = _shares_of(x, rng)
        d0, d1, _ = oracle.drelu(s0, s1, 0, m, SEED)
        assert np.array_equal(d0 + d1, (x >= 0).astype(np.int64)), m
        r0, r1, _ = oracle.relu(s0, s1, 0, m, SEED)
        assert np.array_equal(r0 + r1, np.maximum(x, 0)), m


def test_theorem2_low_cut_prunes_small_positives_only():
    """Dropping k low bits (no high cut): errors only for 0 <= x < 2^k (output pruned to zero), and there
    exactly when the low-bit carry is lost; negatives are never turned positive in the usual range (Theorem 2)."""
    rng = np.random.default_rng(22)
    for k in (1, 4, 12, 16, 30):
        x = np.concatenate([rng.integers(-(1 << (k + 3)), 1 << (k + 3), 6000, dtype=np.int64),
                            rng.integers(0, 1 << k, 2000, dtype=np.int64)])
        s0, s1 = _shares_of(x, rng)
        lowmask = np.uint64((1 << k) - 1)
        carry = ((_u64(s0) & lowmask) + (_u64(s1) & lowmask)) >> np.uint64(k)
        d0, d1, _ = oracle.drelu(s0, s1, k, 64, SEED)
        d = d0 + d1
        exact = (x >= 0).astype(np.int64)
        small = (x >= 0) & (x < (1 << k))
        assert np.array_equal(d[~small], exact[~small])
        assert np.array_equal(d[small], 1 - carry[small].astype(np.int64))
        r0, r1, _ = oracle.relu(s0, s1, k, 64, SEED)
        pruned = np.where(small & (carry == 1), 0, np.maximum(x, 0))
        assert np.array_equal(r0 + r1, pruned)
        assert (carry[small] == 1).any() and (carry[small] == 0).any()


# ----------------------------------------------------------------------------------------------
# brute force on the 8-bit ring: every share pair, every (k, m)
# ----------------------------------------------------------------------------------------------

@pytest.mark.parametrize("variant", [0, 1])
def test_brute_force_ring8_error_set(variant):
    N = 8
    v = np.arange(256, dtype=np.int64)
    s0, s1 = [a.reshape(-1) for a in np.meshgrid(v, v, indexing="ij")]
    xs = (s0 + s1) & 255
    x = np.where(xs >= 128, xs - 256, xs)            # the secret as a signed 8-bit value
    exact = (x >= 0).astype(np.int64)
    checked = 0
    for k in range(N):
        for m in range(k + 1, N + 1):
            w = m - k
            d0, d1, _ = oracle.drelu(s0, s1, k, m, SEED, ring_bits=N, variant=variant)
            d = (d0 + d1) & 255
            assert set(np.unique(d)) <= {0, 1}
            r0, r1, _ = oracle.relu(s0, s1, k, m, SEED, ring_bits=N, variant=variant)
            r = (r0 + r1) & 255
            assert np.array_equal(r, (xs * d) & 255)

            c = (((s0 & ((1 << k) - 1)) + (s1 & ((1 << k) - 1))) >> k).astype(np.int64)   # lost low carry
            # what the slices encode: floor(x' / 2^k) - c on Z_2^w, x' = x mod 2^m
            xm = xs & ((1 << m) - 1)
            enc = ((xm >> k) - c) & ((1 << w) - 1)
            assert np.array_equal(d, 1 - (enc >> (w - 1)))

            half, low = 1 << (m - 1), 1 << k
            sure_pos = (x >= low) & (x < half)
            sure_neg = (x >= -half + low) & (x < 0)
            small = (x >= 0) & (x < low) & (x < half)
            under = (x >= -half) & (x < -half + low) & (x < 0)
            outside = (x < -half) | (x >= half)
            assert np.array_equal(d[sure_pos], np.ones(sure_pos.sum(), dtype=np.int64))
            assert np.array_equal(d[sure_neg], np.zeros(sure_neg.sum(), dtype=np.int64))
            assert np.array_equal(d[small], 1 - c[small])           # pruned iff the carry was dropped
            if w > 1:
                assert np.array_equal(d[under], c[under])           # underflow: wrong iff carry dropped
            # outside the window the sign of (x mod 2^m), read as an m-bit number, is what comes out
            xsig = np.where(xm >= half, xm - (1 << m), xm)
            ok = outside & (xsig >= low) & (xsig < half)
            assert np.array_equal(d[ok], np.ones(ok.sum(), dtype=np.int64))
            # ReLU equals max(x, 0) wherever DReLU is right
            right = d == exact
            assert np.array_equal(r[right], np.maximum(x, 0)[right] & 255)
            # no cut at all: always right
            if (k, m) == (0, N):
                assert right.all()
            # one-sided: a negative x inside the safe window is never called positive
            assert not (d[sure_neg] == 1).any()
            checked += 1
    assert checked == 36


# ----------------------------------------------------------------------------------------------
# host logic of the oracle itself
# ----------------------------------------------------------------------------------------------

def test_range_scatter_and_threads_agree():
    rng = np.random.default_rng(5)
    n = 10007
    s0, s1 = _rand_shares(rng, n)
    for (k, m) in [(12, 20), (0, 64), (8, 14)]:
        a0, a1 = oracle.evaluate(s0, s1, k, m, SEED, oracle.WHAT_RELU)
        t0, t1 = oracle.evaluate(s0, s1, k, m, SEED, oracle.WHAT_RELU, threads=3)
        assert np.array_equal(a0, t0) and np.array_equal(a1, t1)
        idx = rng.choice(n, 500, replace=False).astype(np.uint64)
        g0, g1 = oracle.evaluate_at(s0[idx.astype(np.int64)], s1[idx.astype(np.int64)], idx, k, m, SEED, oracle.WHAT_RELU)
        assert np.array_equal(g0, a0[idx.astype(np.int64)]) and np.array_equal(g1, a1[idx.astype(np.int64)])
        # a window of the tensor evaluated with its global offset
        c0, c1 = oracle.evaluate(s0[1000:2000], s1[1000:2000], k, m, SEED, oracle.WHAT_RELU, first=1000)
        assert np.array_equal(c0, a0[1000:2000]) and np.array_equal(c1, a1[1000:2000])


def test_argument_validation():
    z = np.zeros(4, dtype=np.int64)
    for (k, m) in [(-1, 4), (4, 4), (5, 4), (0, 65), (60, 66)]:
        with pytest.raises(ValueError):
            oracle.drelu(z, z, k, m, SEED)
    with pytest.raises(ValueError):
        oracle.drelu(z, z, 0, 9, SEED, ring_bits=8)
    e = np.zeros(0, dtype=np.int64)
    o0, o1, bits = oracle.relu(e, e, 12, 20, SEED)
    assert o0.size == 0 and o1.size == 0 and bits == 0
    with pytest.raises(ValueError):
        oracle.relu(e, e, 20, 12, SEED)


def test_open_is_add_or_xor():
    rng = np.random.default_rng(9)
    a, b = _rand_shares(rng, 1000)
    assert np.array_equal(oracle.open_shares(a, b), (a.view(np.uint64) + b.view(np.uint64)).view(np.int64))
    assert np.array_equal(oracle.open_shares(a, b, binary=True), a ^ b)
    assert np.array_equal(oracle.open_shares(a, b, ring_bits=8), (a + b) & 255)


def test_output_shares_look_uniform_and_depend_on_seed():
    """The share VALUES are not pinned by the paper; check only what any correct dealer gives: each output
    share alone is (close to) uniform and independent of the secret, and a new seed re-randomises them."""
    rng = np.random.default_rng(33)
    n = 1 << 15
    x = np.rint(rng.standard_normal(n) * 2 * 65536).astype(np.int64)
    s0, s1 = _shares_of(x, rng)
    for what in (oracle.WHAT_DRELU, oracle.WHAT_RELU):
        o0, o1 = oracle.evaluate(s0, s1, 12, 20, SEED, what)
        for o in (o0, o1):
            bits = np.unpackbits(o.view(np.uint8)).mean()
            assert abs(bits - 0.5) < 0.005
            assert abs(np.corrcoef(o.astype(np.float64), x.astype(np.float64))[0, 1]) < 0.03
        p0, p1 = oracle.evaluate(s0, s1, 12, 20, SEED + 1, what)
        assert (p0 != o0).mean() > 0.99
        assert np.array_equal(p0 + p1, o0 + o1)


# ----------------------------------------------------------------------------------------------
# zero-error high-cut scan (Sec. 4.1.2, "eco")
# ----------------------------------------------------------------------------------------------

def _bit_disagreement_counts(x):
    """#{i : bit (m-1) of x_i differs from its sign bit}, m = 1..64 -- what Theorem 1's proof says decides the
    outcome at (0, m): the slices are exact shares of x mod 2^m, so only the sign bit read changes."""
    ux = x.view(np.uint64)
    sign = ux >> np.uint64(63)
    return np.array([int((((ux >> np.uint64(m - 1)) & np.uint64(1)) != sign).sum()) for m in range(1, 65)], dtype=np.uint64)


def test_eco_scan_counts_sign_bit_disagreements():
    rng = np.random.default_rng(41)
    x = np.concatenate([np.rint(rng.standard_normal(700) * 2 * 65536).astype(np.int64),
                        rng.integers(np.iinfo(np.int64).min, np.iinfo(np.int64).max, 100, dtype=np.int64),
                        np.array([0, -1, 1, np.iinfo(np.int64).min, np.iinfo(np.int64).max], dtype=np.int64)])
    s0, s1 = _shares_of(x, rng)
    counts = oracle.eco_scan(s0, s1, seed=SEED)
    assert np.array_equal(counts, _bit_disagreement_counts(x))
    assert counts[63] == 0


def test_eco_choice_is_theorem1_bound():
    """For values in [-2^(t-1), 2^(t-1)) that reach both ends, the zero-error cut is exactly m = t."""
    rng = np.random.default_rng(42)
    for t in (3, 12, 19, 22, 40):
        lo, hi = -(1 << (t - 1)), (1 << (t - 1))
        x = rng.integers(lo, hi, 300, dtype=np.int64)
        x[:2] = [lo, hi - 1]
        s0, s1 = _shares_of(x, rng)
        counts = oracle.eco_scan(s0, s1)
        assert (counts[t - 1:] == 0).all()
        assert counts[t - 2] > 0                       # one bit less already flips the extremes
        assert oracle.eco_choose(counts) == t
    assert oracle.eco_choose(np.zeros(64, dtype=np.uint64)) == 1
    c = np.zeros(64, dtype=np.uint64)
    c[62] = 5
    assert oracle.eco_choose(c) == 64


def test_eco_scan_small_ring_brute_force():
    v = np.arange(256, dtype=np.int64)
    s0, s1 = [a.reshape(-1) for a in np.meshgrid(v, v, indexing="ij")]
    counts = oracle.eco_scan(s0[::7], s1[::7], ring_bits=8)
    xs = (s0[::7] + s1[::7]) & 255
    for m in range(1, 9):
        assert counts[m - 1] == int((((xs >> (m - 1)) & 1) != (xs >> 7)).sum())
    assert (counts[8:] == 0).all()


# ----------------------------------------------------------------------------------------------
# float boundary of the simulator (Sec. 4.1.1; fixed point of Sec. 2.2 / Sec. 3.1)
# ----------------------------------------------------------------------------------------------

def test_float_encode_share_reveal():
    rng = np.random.default_rng(51)
    x = np.concatenate([rng.standard_normal(2000).astype(np.float32) * 3,
                        np.array([0.0, -0.0, 1.5 / 65536, 2.5 / 65536, -1.5 / 65536, -2.5 / 65536, 0.5 / 65536,
                                  1.0, -1.0, 123.456, 2.0 ** 20, -2.0 ** 30], dtype=np.float32)])
    s0, s1 = oracle.share_f32(x, 99)
    # share0 is the generator's output sequence; the shares add up to round-half-even(x * 2^16)
    assert [int(v) & U64 for v in s0[:50]] == oracle.sm_sequence(99, 50)
    enc = (s0.view(np.uint64) + s1.view(np.uint64)).view(np.int64)
    assert np.array_equal(enc, np.rint(x.astype(np.float64) * 65536.0).astype(np.int64))
    assert [int(v) for v in enc[2002:2007]] == [2, 2, -2, -2, 0]           # ties go to even
    y = oracle.reveal_f32(s0, s1)
    assert np.array_equal(y, (enc.astype(np.float64) / 65536.0).astype(np.float32))
    # special values: NaN encodes as 0, huge magnitudes clamp to +-2^62
    sp = np.array([np.nan, np.inf, -np.inf, 3e38, -3e38], dtype=np.float32)
    a, b = oracle.share_f32(sp, 5)
    assert [int(v) for v in (a.view(np.uint64) + b.view(np.uint64)).view(np.int64)] == [0, 1 << 62, -(1 << 62), 1 << 62, -(1 << 62)]


def test_simulated_relu_on_floats():
    """Full ring: exactly ReLU of the quantised input.  Reduced ring: the same wherever the value sits inside the window,
    and small positives may be pruned to zero (Theorem 2) but nothing else changes."""
    rng = np.random.default_rng(52)
    x = (rng.standard_normal(4000) * 2).astype(np.float32)
    q = np.rint(x.astype(np.float64) * 65536.0) / 65536.0
    y = oracle.sim_relu_f32(x, 0, 64, SEED, 1234)
    assert np.array_equal(y, np.maximum(q, 0).astype(np.float32))
    k, m = 12, 20
    y = oracle.sim_relu_f32(x, k, m, SEED, 1234)
    xi = np.rint(x.astype(np.float64) * 65536.0).astype(np.int64)
    inside = (np.abs(xi) < (1 << (m - 1)) - (1 << k))
    big = inside & ((xi >= (1 << k)) | (xi < 0))
    assert np.array_equal(y[big], np.maximum(q, 0).astype(np.float32)[big])
    small = inside & (xi >= 0) & (xi < (1 << k))
    assert np.all((y[small] == 0) | (y[small] == q[small].astype(np.float32)))
    assert (y[small] == 0).any()
