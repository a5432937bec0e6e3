// The protocol among P = 3 or 4 parties, all simulated in one thread (P = 2 is the path of hb_kernels.hpp).
//
// The paper's setting allows any number of parties (Sec. 2.2 "Operation of CrypTen"; Sec. 3.1.2 notes that the
// analysis carries over).  What changes against two parties:
//   - the P sliced shares are summed by a tree of two-operand Kogge-Stone adders on XOR shares:
//     P = 3: (X0 + X1) + X2;  P = 4: (X0 + X1) + (X2 + X3); adders numbered in evaluation order;
//   - an AND gate draws 3P - 1 dealer words a_0..a_{P-1} b_0..b_{P-1} c_0..c_{P-2} (the last c completes a & b);
//   - a group owns (P-1)(1+2R)(3P-1) + 1 words; the last one holds the B2A bits, bit P*j + q = rho_q of lane j;
//   - an element owns 4P - 2 arithmetic words: rA_0..rA_{P-2} | a_0..a_{P-1} | b_0..b_{P-1} | c_0..c_{P-2};
//   - party 0 adds every public term.
//
//   mp_group_kernel   one thread per group, scalar 8-byte accesses: slice widths above 32.
//   mp_tile_kernel    one wavefront per 64 groups (32 below w = 4, where a group has 16 or 21 elements) with
//                     coalesced 16-byte accesses, as tile_kernel: slice widths up to 32.
//
// Algorithmic traffic: 16 P bytes per element.
#pragma once

#include "hb_kernels.hpp"

namespace hb {

constexpr int kMaxParties = 4;

template <int P>
struct Shares {      // one value held as P shares
    uint64_t v[P];
};

struct MpPointers {  // kernel argument: the P input and P output arrays
    const uint64_t *x[kMaxParties];
    uint64_t *o[kMaxParties];
};

template <int W, int P>
struct MpShape {
    static_assert(P >= 3 && P <= kMaxParties, "party count");
    using S = Shape<W>;
    static constexpr int R = S::R;
    static constexpr int L = (64 / W) < (64 / P) ? (64 / W) : (64 / P);   // the B2A word holds P bits per lane
    static constexpr int kGateWords = 3 * P - 1;
    static constexpr int kAdderWords = (1 + 2 * R) * kGateWords;
    static constexpr int kB2aWord = (P - 1) * kAdderWords;
    static constexpr int kWordsPerGroup = kB2aWord + 1;
    static constexpr int kArithWords = 4 * P - 2;
};

// Beaver AND among P parties, returned XORed onto acc share by share; zq = generator state of the gate's first
// dealer word.  As in the two-party gate the operands enter only through the openings: Ux = XOR over the parties
// of U_q, Vx = XOR of V_q before the field mask `keep` of a shifted operand.
template <int P>
__device__ __forceinline__ Shares<P> mp_and(uint64_t zq, uint64_t Ux, uint64_t Vx, uint64_t keep, const Shares<P> &acc)
{
    uint64_t a[P], b[P], c[P];
    uint64_t as = 0, bs = 0, cs = 0;
#pragma unroll
    for (int q = 0; q < P; ++q) {
        a[q] = mix64(zq + (uint64_t)q * kGamma);
        b[q] = mix64(zq + (uint64_t)(P + q) * kGamma);
        as ^= a[q];
        bs ^= b[q];
    }
#pragma unroll
    for (int q = 0; q < P - 1; ++q) {
        c[q] = mix64(zq + (uint64_t)(2 * P + q) * kGamma);
        cs ^= c[q];
    }
    c[P - 1] = bitop3<kTtXorAnd>(cs, as, bs);               // the dealer completes the sharing of c = a & b
    const uint64_t d = Ux ^ as;                             // opened: XOR over the parties of U_q ^ a_q
    const uint64_t e = bitop3<kTtXorAnd>(bs, Vx, keep);     // opened: XOR over the parties of V_q ^ b_q
    Shares<P> Z;
    // party 0 takes the public d & e term: c_0 ^ (d & b_0) ^ (e & a_0) ^ (d & e)
    Z.v[0] = bitop3<kTtXor3>(acc.v[0], bitop3<kTtXorAnd>(c[0], e, a[0]), bitop3<kTtAndXor>(d, b[0], e));
#pragma unroll
    for (int q = 1; q < P; ++q) Z.v[q] = bitop3<kTtXorAnd>(bitop3<kTtXorAnd>(acc.v[q] ^ c[q], d, b[q]), e, a[q]);
    return Z;
}

// X + Y mod 2^W in every field, on XOR shares; za = generator state of the adder's first dealer word.
// The last round's P-update gate is not evaluated (nothing reads it; its words are never drawn).
template <int W, int P>
__device__ __forceinline__ Shares<P> mp_add(uint64_t za, const Shares<P> &X, const Shares<P> &Y)
{
    using S = Shape<W>;
    using M = MpShape<W, P>;
    Shares<P> Pw, Sum, zero;
    uint64_t Xx = 0, Yx = 0;
#pragma unroll
    for (int q = 0; q < P; ++q) {
        Pw.v[q] = Sum.v[q] = X.v[q] ^ Y.v[q];
        zero.v[q] = 0;
        Xx ^= X.v[q];
        Yx ^= Y.v[q];
    }
    Shares<P> G = mp_and<P>(za, Xx, Yx, ~0ull, zero);
#pragma unroll
    for (int r = 0; r < S::R; ++r) {
        const int s = 1 << r;
        const uint64_t keep = S::keep(s);
        // shifting is linear: the XOR of the parties' shifted shares is the shifted XOR of their shares
        uint64_t Gx = 0, Px = 0;
#pragma unroll
        for (int q = 0; q < P; ++q) {
            Gx ^= G.v[q];
            Px ^= Pw.v[q];
        }
        // one gate's dealer words at a time (not_before): 3P - 1 live words instead of the whole adder's
        G = mp_and<P>(not_before(za + (uint64_t)((1 + 2 * r) * M::kGateWords) * kGamma, Gx), Px, Gx << s, keep, G);
        if (r + 1 < S::R)
            Pw = mp_and<P>(not_before(za + (uint64_t)((2 + 2 * r) * M::kGateWords) * kGamma, G.v[0]), Px, Px << s, keep, zero);
    }
    const uint64_t keep1 = S::keep(1);
    Shares<P> out;
#pragma unroll
    for (int q = 0; q < P; ++q) out.v[q] = Sum.v[q] ^ ((G.v[q] << 1) & keep1);
    return out;
}

// XOR shares of (u_0 + ... + u_{P-1}) mod 2^W for one group; zg = generator state of the group's first word.
template <int W, int P>
__device__ __forceinline__ Shares<P> mp_a2b_sum(const uint64_t (&u)[P], uint64_t zg)
{
    using M = MpShape<W, P>;
    Shares<P> X[P];
#pragma unroll
    for (int q = 0; q < P; ++q) {
#pragma unroll
        for (int t = 0; t < P; ++t) X[q].v[t] = (t == q) ? u[q] : 0;    // party q shares its slice trivially
    }
    constexpr uint64_t kAdderStride = (uint64_t)M::kAdderWords * kGamma;
    if constexpr (P == 3) {
        const Shares<P> s01 = mp_add<W, P>(zg, X[0], X[1]);
        return mp_add<W, P>(zg + kAdderStride, s01, X[2]);
    } else {
        const Shares<P> s01 = mp_add<W, P>(zg, X[0], X[1]);
        const Shares<P> s23 = mp_add<W, P>(zg + kAdderStride, X[2], X[3]);
        return mp_add<W, P>(zg + 2 * kAdderStride, s01, s23);
    }
}

// Everything after the circuit for one element.  sign / rho: bit q = party q's XOR share of the sign / of the
// dealer bit.  zA = generator state of the element's first arithmetic word.  MODE: kDrelu or kRelu.
template <int P, int MODE>
__device__ __forceinline__ Shares<P> mp_finish(uint32_t sign, uint32_t rho, const Shares<P> &x, uint64_t zA)
{
    const uint64_t z = (uint64_t)(__popc(sign ^ rho) & 1);    // opened bit
    const uint64_t r = (uint64_t)(__popc(rho) & 1);           // known to the dealer only
    uint64_t rA[P], rsum = 0;
#pragma unroll
    for (int q = 0; q < P - 1; ++q) {
        rA[q] = mix64(zA + (uint64_t)q * kGamma);
        rsum += rA[q];
    }
    rA[P - 1] = r - rsum;
    Shares<P> D;
#pragma unroll
    for (int q = 0; q < P; ++q) {
        const uint64_t pub = (q == 0) ? 1 : 0;
        const uint64_t beta = z ? (pub - rA[q]) : rA[q];       // sign = z + r - 2zr, party 0 adds the public z
        D.v[q] = pub - beta;
    }
    if (MODE == kDrelu) return D;

    const uint64_t zM = zA + (uint64_t)(P - 1) * kGamma;
    uint64_t a[P], b[P], c[P];
    uint64_t as = 0, bs = 0, cs = 0, xs = 0, del = 0;
#pragma unroll
    for (int q = 0; q < P; ++q) {
        a[q] = mix64(zM + (uint64_t)q * kGamma);
        b[q] = mix64(zM + (uint64_t)(P + q) * kGamma);
        as += a[q];
        bs += b[q];
        xs += x.v[q];
        del += D.v[q] - b[q];                // opened: each party's message D_q - b_q, summed
    }
#pragma unroll
    for (int q = 0; q < P - 1; ++q) {
        c[q] = mix64(zM + (uint64_t)(2 * P + q) * kGamma);
        cs += c[q];
    }
    const uint64_t eps = xs - as;            // opened: sum over the parties of x_q - a_q
    Shares<P> out;
    // party 0 takes the public term: c_0 + eps * b_0 + del * a_0 + eps * del
    out.v[0] = sum_of_products(c[0], eps, b[0] + del, del, a[0]);
#pragma unroll
    for (int q = 1; q < P - 1; ++q) out.v[q] = sum_of_products(c[q], eps, b[q], del, a[q]);
    // the last party's c completes the triple: c_{P-1} = a * b - (c_0 + ... + c_{P-2})
    out.v[P - 1] = sum_of_products(0 - cs, as, bs, eps, b[P - 1], del, a[P - 1]);
    return out;
}

template <int W, int P, int MODE>
__global__ void __launch_bounds__(kBlock)
mp_group_kernel(const MpPointers ptr, uint64_t n, uint64_t groups, int k, uint64_t seedB, uint64_t seedA)
{
    using S = Shape<W>;
    using M = MpShape<W, P>;
    constexpr int L = M::L;
    const uint64_t g = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (g >= groups) return;
    const uint64_t i0 = g * (uint64_t)L;
    const int cnt = (n - i0) >= (uint64_t)L ? L : (int)(n - i0);

    uint64_t u[P];
#pragma unroll
    for (int q = 0; q < P; ++q) u[q] = 0;
#pragma unroll
    for (int j = 0; j < L; ++j) {
        if (j < cnt) {
#pragma unroll
            for (int q = 0; q < P; ++q) u[q] |= ((load_stream(ptr.x[q] + i0 + j) >> k) & S::kField) << (j * W % 64);
        }
    }
    const uint64_t zg = seedB + (g * (uint64_t)M::kWordsPerGroup + 1) * kGamma;
    const Shares<P> sum = mp_a2b_sum<W, P>(u, zg);
    const uint64_t wb = mix64(zg + (uint64_t)M::kB2aWord * kGamma);

#pragma unroll
    for (int j = 0; j < L; ++j) {
        if (j < cnt) {
            uint32_t sign = 0;
            Shares<P> x;
#pragma unroll
            for (int q = 0; q < P; ++q) {
                sign |= (uint32_t)((sum.v[q] >> (j * W + W - 1)) & 1) << q;
                x.v[q] = (MODE == kRelu) ? load_stream(ptr.x[q] + i0 + j) : 0;
            }
            const uint32_t rho = (uint32_t)(wb >> (P * j)) & ((1u << P) - 1);
            const uint64_t zA = seedA + ((uint64_t)M::kArithWords * (i0 + j) + 1) * kGamma;
            const Shares<P> out = mp_finish<P, MODE>(sign, rho, x, zA);
#pragma unroll
            for (int q = 0; q < P; ++q) store_stream(ptr.o[q] + i0 + j, out.v[q]);
        }
    }
}

// Tile kernel among P parties: the owner / group-lane scheme of tile_body.  LDS per wavefront: P arrays of one
// entry (1, 2 or 4 bytes) per element for the slices, and per group {sign shares, B2A word}; the sign share of
// party q for lane j sits at bit j*W + q when a field has room for P bits (W >= P); narrower fields publish one
// word per party instead (the sum word itself: the sign of lane j is bit j*W + W - 1).
template <int W, int P>
struct MpTileTraits {
    using M = MpShape<W, P>;
    static constexpr int L = M::L;
    static constexpr bool kSupported = (W <= 32);
    static constexpr int kGroups = (W >= 4) ? kWave : kWave / 2;   // half the lanes run the circuit when L > 16:
    static constexpr int kTile = kGroups * L;                      // a lane then owns at most 6 element pairs
    static constexpr int kPairs = (kTile / 2 + kWave - 1) / kWave;
    static constexpr bool kSignWords = (W < P);
    using Entry = typename std::conditional<(W <= 8), uint8_t,
                  typename std::conditional<(W <= 16), uint16_t, uint32_t>::type>::type;
    static constexpr bool kWordIsPacked = (int)sizeof(Entry) * 8 == W;   // the L entries of a group are its SWAR word
    static constexpr int kSliceBytes = ((kTile * (int)sizeof(Entry) + 15) / 16) * 16;   // per party
};

// Work of one wavefront on wave-tile `tile` (uniform over the wavefront).  FULL: the whole tile lies inside the
// tensor, so no access needs a bounds check (every tile but the last).
template <int W, int P, int MODE, bool FULL>
__device__ __forceinline__ void mp_tile_body(const MpPointers &ptr, uint64_t n, int k, uint64_t seedB, uint64_t seedA,
                                             uint64_t tile, int lane, unsigned char (*slice_lds)[MpTileTraits<W, P>::kSliceBytes],
                                             U64x2 *verdict, uint64_t (*sign_words)[P])
{
    using S = Shape<W>;
    using M = MpShape<W, P>;
    using T = MpTileTraits<W, P>;
    using Entry = typename T::Entry;
    constexpr int L = T::L;
    const uint64_t tile0 = tile * T::kTile;

    // ---- owners: load, slice, deposit
    U64x2 xs[P][T::kPairs];
#pragma unroll
    for (int c = 0; c < T::kPairs; ++c) {
        const unsigned e = 2 * (c * kWave + lane);
#pragma unroll
        for (int q = 0; q < P; ++q) xs[q][c] = U64x2{0, 0};
        if (e < (unsigned)T::kTile) {
#pragma unroll
            for (int q = 0; q < P; ++q) {
                const uint64_t *t = ptr.x[q] + tile0;       // scalar base, 32-bit lane offset
                if (FULL || tile0 + e + 1 < n) {
                    xs[q][c] = load_stream2(t + e);
                } else if (tile0 + e < n) {
                    xs[q][c].a = load_stream(t + e);
                }
                Entry *sl = reinterpret_cast<Entry *>(slice_lds[q]);
                sl[e] = (Entry)((xs[q][c].a >> k) & S::kField);
                sl[e + 1] = (Entry)((xs[q][c].b >> k) & S::kField);
            }
        }
    }
    wave_sync();

    // ---- group lanes: collect the fields of group `lane`, run the adder tree, publish signs and B2A word
    if (T::kGroups == kWave || lane < T::kGroups) {
        uint64_t u[P];
#pragma unroll
        for (int q = 0; q < P; ++q) {
            if constexpr (T::kWordIsPacked) {
                u[q] = reinterpret_cast<const uint64_t *>(slice_lds[q])[lane];
            } else {
                const Entry *sl = reinterpret_cast<const Entry *>(slice_lds[q]);
                u[q] = 0;
#pragma unroll
                for (int j = 0; j < L; ++j) u[q] |= (uint64_t)sl[lane * L + j] << (j * W);
            }
        }
        const uint64_t g = tile * T::kGroups + lane;
        const uint64_t zg = seedB + (g * (uint64_t)M::kWordsPerGroup + 1) * kGamma;
        const Shares<P> sum = mp_a2b_sum<W, P>(u, zg);
        const uint64_t ones = S::ones();
        uint64_t sg = 0;
        if constexpr (T::kSignWords) {
#pragma unroll
            for (int q = 0; q < P; ++q) sign_words[lane][q] = sum.v[q];
        } else {
#pragma unroll
            for (int q = 0; q < P; ++q) sg |= ((sum.v[q] >> (W - 1)) & ones) << q;
        }
        verdict[lane] = U64x2{sg, mix64(zg + (uint64_t)M::kB2aWord * kGamma)};
    }
    wave_sync();

    // ---- owners: pick up the verdict of each element's group, finish, store
    const uint64_t zA0 = seedA + ((uint64_t)M::kArithWords * (tile0 + 2 * (uint64_t)lane) + 1) * kGamma;
#pragma unroll
    for (int c = 0; c < T::kPairs; ++c) {
        const unsigned e = 2 * (c * kWave + lane);
        if (e < (unsigned)T::kTile) {
            const int grp0 = e / L, j0 = e - grp0 * L;
            const U64x2 v0 = verdict[grp0];
            const bool split = (L % 2 != 0) && (j0 == L - 1);     // the pair straddles two groups (odd L only)
            const U64x2 v1 = split ? verdict[grp0 + 1] : v0;
            Shares<P> r[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const U64x2 v = h ? v1 : v0;
                const int j = h ? (split ? 0 : j0 + 1) : j0;
                uint32_t sign;
                if constexpr (T::kSignWords) {
                    const int gj = h ? (split ? grp0 + 1 : grp0) : grp0;
                    sign = 0;
#pragma unroll
                    for (int q = 0; q < P; ++q) sign |= ((uint32_t)(sign_words[gj][q] >> (j * W + W - 1)) & 1u) << q;
                } else {
                    sign = (uint32_t)(v.a >> (j * W)) & ((1u << P) - 1);
                }
                const uint32_t rho = (uint32_t)(v.b >> (P * j)) & ((1u << P) - 1);
                Shares<P> x;
#pragma unroll
                for (int q = 0; q < P; ++q) x.v[q] = h ? xs[q][c].b : xs[q][c].a;
                const uint64_t zA = zA0 + (uint64_t)(M::kArithWords * (2 * c * kWave + h)) * kGamma;
                r[h] = mp_finish<P, MODE>(sign, rho, x, zA);
            }
#pragma unroll
            for (int q = 0; q < P; ++q) {
                uint64_t *t = ptr.o[q] + tile0;
                if (FULL || tile0 + e + 1 < n) {
                    store_stream2(t + e, U64x2{r[0].v[q], r[1].v[q]});
                } else if (tile0 + e < n) {
                    store_stream(t + e, r[0].v[q]);
                }
            }
        }
    }
}

template <int W, int P, int MODE>
__global__ void __launch_bounds__(kBlock)
mp_tile_kernel(const MpPointers ptr, uint64_t n, int k, uint64_t seedB, uint64_t seedA)
{
    using T = MpTileTraits<W, P>;
    static_assert(T::kSupported, "tile kernel needs W <= 32");
    __shared__ __attribute__((aligned(16))) unsigned char slices_all[kWavesPerBlock][P][T::kSliceBytes];
    __shared__ U64x2 verdict_all[kWavesPerBlock][kWave];
    __shared__ uint64_t sign_words_all[kWavesPerBlock][T::kSignWords ? kWave : 1][P];
    const int lane = threadIdx.x % kWave, wv = wave_index();
    const uint64_t tile = (uint64_t)blockIdx.x * kWavesPerBlock + wv;
    if (tile * T::kTile >= n) return;        // whole wavefront beyond the tensor
    if ((tile + 1) * T::kTile <= n)
        mp_tile_body<W, P, MODE, true>(ptr, n, k, seedB, seedA, tile, lane, slices_all[wv], verdict_all[wv], sign_words_all[wv]);
    else
        mp_tile_body<W, P, MODE, false>(ptr, n, k, seedB, seedA, tile, lane, slices_all[wv], verdict_all[wv], sign_words_all[wv]);
}

}  // namespace hb
