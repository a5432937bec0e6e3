// Device-side statement of the protocol, in SWAR form: L = min(64/W, 32) elements share one 64-bit word,
// element j of a group occupying bits [jW, jW+W).  Every step below is bitwise, so the L fields never
// interact except through shifts, which are confined to their field by a mask.
//
// Paper: Sec. 2.2 "Evaluating ReLU with GMW" (A2B adder on XOR shares, Beaver AND, sign, B2A),
// Eq. 3 (DReLU on the slice only), Sec. 4.2 (depth ceil(log2 w), packing of w-bit fields in 64-bit words).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hb {

// ---- dealer streams: SplitMix64, output j of a generator started at state s is mix(s + (j+1)*gamma)
constexpr uint64_t kGamma = 0x9E3779B97F4A7C15ull;

__host__ __device__ __forceinline__ uint64_t mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__host__ __device__ __forceinline__ uint64_t stream_word(uint64_t s, uint64_t j)
{
    return mix64(s + (j + 1) * kGamma);
}

// ---- compile-time shape of the circuit for slice width W
constexpr int ceil_log2(int w)
{
    int r = 0;
    while ((1 << r) < w) ++r;
    return r;
}

template <int W>
struct Shape {
    static_assert(W >= 1 && W <= 64, "slice width");
    static constexpr int w = W;
    static constexpr int R = ceil_log2(W);                     // prefix rounds (0 when W == 1)
    static constexpr int L = (64 / W) > 32 ? 32 : (64 / W);     // fields per word
    static constexpr int kGates = 1 + 2 * R;                    // gate 0 + two per round

    // Dealer words of one group.  Standard layout: five triple words (a_0 a_1 b_0 b_1 c_0) per gate, then the
    // B2A word.  Shared-mask layout: gate 0 as before; a prefix round owns eight words, a_0 a_1 (the one mask of
    // P that both of its gates use), b_0 b_1 c_0 of the G-update and b_0 b_1 c_0 of the P-update; then the B2A word.
    static constexpr int round_word(bool shared, int r) { return shared ? 5 + 8 * r : 5 * (1 + 2 * r); }
    static constexpr int b2a_word(bool shared) { return round_word(shared, R); }
    static constexpr int words_per_group(bool shared) { return b2a_word(shared) + 1; }
    static constexpr uint64_t kField = (W == 64) ? ~0ull : ((1ull << (W & 63)) - 1);

    // bit 0 of every field
    static constexpr uint64_t ones()
    {
        uint64_t r = 0;
        for (int j = 0; j < L; ++j) r |= 1ull << (j * W);
        return r;
    }
    // positions of a word that still hold data of their own field after a left shift by s
    static constexpr uint64_t keep(int s)
    {
        uint64_t f = (s >= W) ? 0 : ((kField << s) & kField);
        uint64_t r = 0;
        for (int j = 0; j < L; ++j) r |= f << (j * W);
        return r;
    }
};

struct Pair {      // one value held as (party 0 share, party 1 share)
    uint64_t p0, p1;
};

// Returns z, which the compiler may not compute before `after` is known.  Dealer words depend only on the group
// or element number, so the scheduler would otherwise generate those of every gate ahead of the circuit and
// hold them all in registers; tying a gate's generator state to the previous gate's result keeps their live
// ranges one gate long.  Emits no instruction.
__device__ __forceinline__ uint64_t not_before(uint64_t z, uint64_t after)
{
    asm("" : "+v"(z) : "v"(after));
    return z;
}

// ---- three-input bitwise operations (v_bitop3_b32, one instruction per 32-bit half) ----------------------------
// The 8-bit truth table of a boolean function f(a, b, c), in the instruction's operand order.
constexpr unsigned kTtXor3 = (0xF0 ^ 0xCC ^ 0xAA) & 0xFF;              // a ^ b ^ c
constexpr unsigned kTtXorAnd = (0xF0 ^ (0xCC & 0xAA)) & 0xFF;          // a ^ (b & c)
constexpr unsigned kTtAndXor = (0xF0 & (0xCC ^ 0xAA)) & 0xFF;          // a & (b ^ c)

template <unsigned TT>
__device__ __forceinline__ uint64_t bitop3(uint64_t a, uint64_t b, uint64_t c)
{
    const uint32_t lo = __builtin_amdgcn_bitop3_b32((uint32_t)a, (uint32_t)b, (uint32_t)c, TT);
    const uint32_t hi = __builtin_amdgcn_bitop3_b32((uint32_t)(a >> 32), (uint32_t)(b >> 32), (uint32_t)(c >> 32), TT);
    return ((uint64_t)hi << 32) | lo;
}

struct GateWords {   // the five dealer words of one AND gate, in stream order
    uint64_t a0, a1, b0, b1, c0;
};

// One Beaver AND on XOR-shared words, Z = U & V, returned as acc ^ Z share by share (acc = {0, 0} for the
// plain gate; the G-update of a prefix round passes the old G).  U is masked by a, V by b.
// The gate sees U and V only through the two openings, and an opening is the XOR of what the two parties
// send, (U_0 ^ a_0) ^ (U_1 ^ a_1) = (U_0 ^ U_1) ^ (a_0 ^ a_1); the caller passes Ux = U_0 ^ U_1 and
// Vx = (V_0 ^ V_1) before the field mask `keep` that confines a shifted operand to its field (all ones when
// the operand is not shifted).  Party 0 takes the public d & e term.
__device__ __forceinline__ Pair beaver_and_words(const GateWords &t, uint64_t Ux, uint64_t Vx, uint64_t keep, Pair acc)
{
    const uint64_t a0 = t.a0, a1 = t.a1, b0 = t.b0, b1 = t.b1, c0 = t.c0;
    const uint64_t a = a0 ^ a1, b = b0 ^ b1;                    // the dealer's triple (a, b, a & b)
    const uint64_t d = Ux ^ a;                                  // opened
    const uint64_t e = bitop3<kTtXorAnd>(b, Vx, keep);          // opened: (Vx & keep) ^ b
    Pair Z;
    // party 0: acc ^ c_0 ^ (e & a_0) ^ (d & (b_0 ^ e))    [= c_0 ^ (d & b_0) ^ (e & a_0) ^ (d & e)]
    Z.p0 = bitop3<kTtXor3>(acc.p0, bitop3<kTtXorAnd>(c0, e, a0), bitop3<kTtAndXor>(d, b0, e));
    // party 1: acc ^ c_1 ^ (d & b_1) ^ (e & a_1), the dealer having completed c_1 = (a & b) ^ c_0
    const uint64_t c1 = bitop3<kTtXorAnd>(c0, a, b);
    Z.p1 = bitop3<kTtXorAnd>(bitop3<kTtXorAnd>(acc.p1 ^ c1, d, b1), e, a1);
    return Z;
}

// The same gate drawing its words inline: zq is the generator state of the gate's first dealer word; the five
// words a_0 a_1 b_0 b_1 c_0 are consecutive outputs.
__device__ __forceinline__ Pair beaver_and(uint64_t zq, uint64_t Ux, uint64_t Vx, uint64_t keep, Pair acc)
{
    GateWords t;
    t.a0 = mix64(zq);
    t.a1 = mix64(zq + 1 * kGamma);
    t.b0 = mix64(zq + 2 * kGamma);
    t.b1 = mix64(zq + 3 * kGamma);
    t.c0 = mix64(zq + 4 * kGamma);
    return beaver_and_words(t, Ux, Vx, keep, acc);
}

// The two Beaver ANDs of a prefix round when one mask serves their common first operand U: T = U & V, Q = U & Y.
// zr is the generator state of the round's first word; the eight words a_0 a_1 | b_0 b_1 c_0 (for V) |
// b_0 b_1 c_0 (for Y) are consecutive outputs.  d = U ^ a is opened once.  Operands and `keep` as in beaver_and;
// T comes back XORed onto accT.  With kSecond false only the first gate is evaluated and its three last words are
// never drawn.
template <bool kSecond>
__device__ __forceinline__ void beaver_and_shared(uint64_t zr, uint64_t Ux, uint64_t Vx, uint64_t Yx, uint64_t keep,
                                                  Pair accT, Pair &T, Pair &Q)
{
    const uint64_t a0 = mix64(zr);
    const uint64_t a1 = mix64(zr + 1 * kGamma);
    const uint64_t a = a0 ^ a1;
    const uint64_t d = Ux ^ a;
    {
        const uint64_t b0 = mix64(zr + 2 * kGamma);
        const uint64_t b1 = mix64(zr + 3 * kGamma);
        const uint64_t c0 = mix64(zr + 4 * kGamma);
        const uint64_t b = b0 ^ b1;
        const uint64_t e = bitop3<kTtXorAnd>(b, Vx, keep);
        T.p0 = bitop3<kTtXor3>(accT.p0, bitop3<kTtXorAnd>(c0, e, a0), bitop3<kTtAndXor>(d, b0, e));
        const uint64_t c1 = bitop3<kTtXorAnd>(c0, a, b);
        T.p1 = bitop3<kTtXorAnd>(bitop3<kTtXorAnd>(accT.p1 ^ c1, d, b1), e, a1);
    }
    if (kSecond) {
        const uint64_t b0 = mix64(zr + 5 * kGamma);
        const uint64_t b1 = mix64(zr + 6 * kGamma);
        const uint64_t c0 = mix64(zr + 7 * kGamma);
        const uint64_t b = b0 ^ b1;
        const uint64_t e = bitop3<kTtXorAnd>(b, Yx, keep);
        Q.p0 = bitop3<kTtXorAnd>(c0, e, a0) ^ bitop3<kTtAndXor>(d, b0, e);
        const uint64_t c1 = bitop3<kTtXorAnd>(c0, a, b);
        Q.p1 = bitop3<kTtXorAnd>(bitop3<kTtXorAnd>(c1, d, b1), e, a1);
    }
}

// A2B + sign for one group.  u0/u1: the L sliced shares of party 0 / party 1 packed as fields.
// zg: generator state of the group's first dealer word.  Returns XOR shares of the sum word
// S ^ (G << 1); the sign of field j is bit jW + W - 1.  The last round's P-update gate is not
// evaluated: nothing reads its result (its dealer words are simply never drawn).  SHARED selects the
// dealer layout in which the two gates of a round share the mask of P.
template <int W, bool SHARED>
__device__ __forceinline__ Pair a2b_sum(uint64_t u0, uint64_t u1, uint64_t zg)
{
    using S = Shape<W>;
    // X = (u0, 0), Y = (0, u1): each party XOR-shares its own slice trivially
    const Pair X{u0, 0}, Y{0, u1};
    Pair P{X.p0 ^ Y.p0, X.p1 ^ Y.p1};
    const Pair Sum = P;
    Pair G = beaver_and(zg, X.p0 ^ X.p1, Y.p0 ^ Y.p1, ~0ull, Pair{0, 0});
#pragma unroll
    for (int r = 0; r < S::R; ++r) {
        const int s = 1 << r;
        const uint64_t keep = S::keep(s);
        // shifting is linear: the XOR of the parties' shifted shares is the shifted XOR of their shares
        const uint64_t Px = P.p0 ^ P.p1;
        const uint64_t Gsx = (G.p0 ^ G.p1) << s, Psx = Px << s;
        const uint64_t zr = not_before(zg + (uint64_t)S::round_word(SHARED, r) * kGamma, G.p0);
        if (SHARED) {
            Pair Pn = P;
            if (r + 1 < S::R) beaver_and_shared<true>(zr, Px, Gsx, Psx, keep, G, G, Pn);
            else beaver_and_shared<false>(zr, Px, Gsx, Psx, keep, G, G, Pn);
            P = Pn;
        } else {
            G = beaver_and(zr, Px, Gsx, keep, G);
            if (r + 1 < S::R) P = beaver_and(zr + 5 * kGamma, Px, Psx, keep, Pair{0, 0});
        }
    }
    const uint64_t keep1 = S::keep(1);
    return Pair{Sum.p0 ^ ((G.p0 << 1) & keep1), Sum.p1 ^ ((G.p1 << 1) & keep1)};
}

// The same circuit on dealer words that were generated elsewhere (standard layout): words[5q + s] is slot s of
// gate q for q = 0 .. 2R - 1 (the last round's P-update gate, q = 2R, is not evaluated and has no entry).
template <int W>
__device__ __forceinline__ Pair a2b_sum_words(uint64_t u0, uint64_t u1, const uint64_t *words)
{
    using S = Shape<W>;
    auto gate = [&](int q) { return GateWords{words[5 * q], words[5 * q + 1], words[5 * q + 2], words[5 * q + 3], words[5 * q + 4]}; };
    const Pair X{u0, 0}, Y{0, u1};
    Pair P{X.p0 ^ Y.p0, X.p1 ^ Y.p1};
    const Pair Sum = P;
    Pair G = beaver_and_words(gate(0), X.p0 ^ X.p1, Y.p0 ^ Y.p1, ~0ull, Pair{0, 0});
#pragma unroll
    for (int r = 0; r < S::R; ++r) {
        const int s = 1 << r;
        const uint64_t keep = S::keep(s);
        const uint64_t Px = P.p0 ^ P.p1;
        const uint64_t Gsx = (G.p0 ^ G.p1) << s, Psx = Px << s;
        G = beaver_and_words(gate(1 + 2 * r), Px, Gsx, keep, G);
        if (r + 1 < S::R) P = beaver_and_words(gate(2 + 2 * r), Px, Psx, keep, Pair{0, 0});
    }
    const uint64_t keep1 = S::keep(1);
    return Pair{Sum.p0 ^ ((G.p0 << 1) & keep1), Sum.p1 ^ ((G.p1 << 1) & keep1)};
}

// B2A of the sign bit and 1 - sign, for one element.  sign/rho: XOR shares of the sign and of the
// dealer bit r.  zA: generator state of the element's first arithmetic word A[6i].
__device__ __forceinline__ Pair b2a_drelu(Pair sign, Pair rho, uint64_t zA)
{
    const uint64_t z = (sign.p0 ^ rho.p0) ^ (sign.p1 ^ rho.p1);   // opened bit
    const uint64_t r = rho.p0 ^ rho.p1;                           // known to the dealer only
    const uint64_t rA0 = mix64(zA);
    const uint64_t rA1 = r - rA0;
    // sign = z ^ r = z + r - 2zr; party 0 adds the public z
    const uint64_t beta0 = z ? (1 - rA0) : rA0;
    const uint64_t beta1 = z ? (0 - rA1) : rA1;
    return Pair{1 - beta0, 0 - beta1};
}

// ---- products on Z_2^64 out of 32-bit halves --------------------------------------------------------------------
// x * y mod 2^64 = lo(x) lo(y) + 2^32 (lo(x) hi(y) + hi(x) lo(y)).  v_mad_u64_u32 (32 x 32 + 64 -> 64) adds while it
// multiplies, so a sum of products costs one instruction per 32 x 32 product plus one final add when the cross
// products are accumulated in a 64-bit register of their own, of which only the low half is used.  held() keeps
// that register whole: without it the compiler narrows the chain to 32-bit multiplies followed by separate adds.
__device__ __forceinline__ uint64_t held(uint64_t v)
{
    asm("" : "+v"(v));
    return v;
}
__device__ __forceinline__ uint64_t lo32(uint64_t v) { return (uint32_t)v; }
__device__ __forceinline__ uint64_t hi32(uint64_t v) { return v >> 32; }
// low + 2^32 * cross, touching only the high half of `low`
__device__ __forceinline__ uint64_t add_to_high(uint64_t low, uint64_t cross)
{
    uint32_t h = (uint32_t)(low >> 32) + (uint32_t)cross;
    asm("" : "+v"(h));      // keeps the sum a 32-bit add (otherwise it is widened to a 64-bit add of {0, cross})
    return ((uint64_t)h << 32) | (uint32_t)low;
}

// acc + x * y (+ u * v) (+ s * t)  mod 2^64
__device__ __forceinline__ uint64_t sum_of_products(uint64_t acc, uint64_t x, uint64_t y, uint64_t u, uint64_t v)
{
    uint64_t cross = held(lo32(x) * hi32(y));
    cross = held(hi32(x) * lo32(y) + cross);
    cross = held(lo32(u) * hi32(v) + cross);
    cross = held(hi32(u) * lo32(v) + cross);
    const uint64_t low = lo32(u) * lo32(v) + (lo32(x) * lo32(y) + acc);
    return add_to_high(held(low), cross);
}
__device__ __forceinline__ uint64_t sum_of_products(uint64_t acc, uint64_t x, uint64_t y, uint64_t u, uint64_t v,
                                                    uint64_t s, uint64_t t)
{
    uint64_t cross = held(lo32(x) * hi32(y));
    cross = held(hi32(x) * lo32(y) + cross);
    cross = held(lo32(u) * hi32(v) + cross);
    cross = held(hi32(u) * lo32(v) + cross);
    cross = held(lo32(s) * hi32(t) + cross);
    cross = held(hi32(s) * lo32(t) + cross);
    const uint64_t low = lo32(s) * lo32(t) + (lo32(u) * lo32(v) + (lo32(x) * lo32(y) + acc));
    return add_to_high(held(low), cross);
}

// Beaver multiply x * D on Z_2^64 for one element; the triple is A[6i+1 .. 6i+5].
__device__ __forceinline__ Pair beaver_mul(Pair x, Pair D, uint64_t zA)
{
    const uint64_t a0 = mix64(zA + 1 * kGamma);
    const uint64_t a1 = mix64(zA + 2 * kGamma);
    const uint64_t b0 = mix64(zA + 3 * kGamma);
    const uint64_t b1 = mix64(zA + 4 * kGamma);
    const uint64_t c0 = mix64(zA + 5 * kGamma);
    const uint64_t a = a0 + a1, b = b0 + b1;                      // the dealer's triple (a, b, a * b)
    const uint64_t eps = (x.p0 + x.p1) - a;                       // opened: (x_0 - a_0) + (x_1 - a_1)
    const uint64_t del = (D.p0 - b0) + (D.p1 - b1);               // opened: each party's message, summed
    Pair out;
    // party 0: c_0 + eps * b_0 + del * a_0 + eps * del
    out.p0 = sum_of_products(c0, eps, b0 + del, del, a0);
    // party 1: c_1 + eps * b_1 + del * a_1, the dealer having completed c_1 = a * b - c_0
    out.p1 = sum_of_products(0 - c0, a, b, eps, b1, del, a1);
    return out;
}

// What a launch computes.  The two last modes run the same operation on the shared-mask dealer layout.
enum Mode { kDrelu = 0, kRelu = 1, kSign = 2, kDreluShared = 3, kReluShared = 4, kModes = 5 };

constexpr int op_of(int mode) { return mode >= kDreluShared ? mode - kDreluShared : mode; }
constexpr bool shared_of(int mode) { return mode >= kDreluShared; }

// Everything after the circuit for element j of a group: pick the element's sign and dealer bits
// out of the group words, B2A, multiply.
template <int W, int MODE>
__device__ __forceinline__ Pair finish_element(Pair sum, uint64_t wb, int j, Pair x, uint64_t zA)
{
    const int sb = j * W + W - 1;
    const Pair sign{(sum.p0 >> sb) & 1, (sum.p1 >> sb) & 1};
    if (op_of(MODE) == kSign) return sign;
    const Pair rho{(wb >> (2 * j)) & 1, (wb >> (2 * j + 1)) & 1};
    const Pair D = b2a_drelu(sign, rho, zA);
    if (op_of(MODE) == kDrelu) return D;
    return beaver_mul(x, D, zA);
}

}  // namespace hb
