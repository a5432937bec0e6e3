// Party-faithful evaluation of one ReLU: every opening of the protocol goes through memory.
//
// The fused kernels keep both parties in one thread and open values in registers.  Here each party is
// a separate set of threads (blockIdx.y = party) that owns its shares, its circuit state and its "wire":
// the packed words it would send to the other party (paper Sec. 2.2: every AND, the B2A and the multiply
// open masked values; Sec. 4.2: the w-bit fields travel packed in 64-bit words, depth ceil(log2 w)).
// A party reads the other party's wire only for rounds that are complete; one kernel launch per
// communication round is the synchronisation, so the launch sequence is the message schedule
//     slice + gate 0  ->  R prefix rounds  ->  sign  ->  B2A bits  ->  multiply openings  ->  result
// and the bytes written to a wire are what a two-GPU run would put on the link.  The result shares are
// bit-identical to the fused kernels'.
//
// Dealer material is generated inline from the same SplitMix64 streams: a party derives its own triple
// shares a_p, b_p, c_p; party 1's c_1 (and r - r^A_0, and the multiply's c_1) needs the whole triple,
// which stands in for the dealer having sent it.
//
// Wire of party p (64-bit words): [2G gate 0][4G per round x R][ceil(n/64) B2A][2n multiply]; field j of a
// group word sits at bit j*w and bits that belong to no element are zero.  The last round's P-update gate
// is opened like every other gate (it is part of the opened-bit count) although nothing consumes its result.
// On the shared-mask dealer layout the two gates of a round have one mask for P, so a round sends three words
// per group (P ^ a once, then the two masked second operands): [3G per round x R].
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hb_protocol.hpp"

namespace hb {

struct PartyShape {
    int w, R, L, k;
    int shared;                 // dealer layout: 0 one triple per gate, 1 one mask of P per round
    int per_round;              // wire words a round sends per group: 4, or 3 on the shared-mask layout
    uint64_t words_per_group;   // 5 (1 + 2R) + 1, or 5 + 8R + 1
    uint64_t field;             // 2^w - 1
    uint64_t ones;              // bit 0 of every field
    uint64_t live;              // all bits of the L fields
    uint64_t keep[6];           // keep[r]: positions still inside their field after << 2^r
    uint64_t keep1;             // same for << 1
};

struct PartyCtx {
    const uint64_t *x[2];
    uint64_t *out[2];
    uint64_t n, groups;
    uint64_t seedB, seedA;
    uint64_t *S[2], *P[2], *G[2], *Z[2];   // per group: sum operand, propagate, generate, masked sign bits (bit j)
    uint64_t *D[2];                        // per element: DReLU share
    uint64_t *wire[2];
    uint64_t off_b2a, off_mul;             // word offsets of the B2A and multiply sections
};

struct PartyTriple {
    uint64_t a, b, c;    // this party's shares of the gate's triple
};

// Party p's shares of the triple of gate q of group g.  Standard layout: gate q owns words 5q .. 5q + 4
// (a_0 a_1 b_0 b_1 c_0).  Shared-mask layout: gate 0 as before; round r owns words 5 + 8r .. 5 + 8r + 7 =
// a_0 a_1 | b_0 b_1 c_0 of its G-update (gate 1 + 2r) | b_0 b_1 c_0 of its P-update (gate 2 + 2r).
__device__ __forceinline__ PartyTriple party_triple(const PartyCtx &c, const PartyShape &s, int p, uint64_t g, int q, bool need_c)
{
    uint64_t wa = 5 * (uint64_t)q, wb = wa + 2;      // word of a_0, word of b_0 (a_1 and b_1, c_0 follow)
    if (s.shared && q > 0) {
        const int r = (q - 1) / 2;
        wa = 5 + 8 * (uint64_t)r;
        wb = wa + (((q - 1) & 1) ? 5 : 2);
    }
    const uint64_t za = c.seedB + (g * s.words_per_group + wa + 1) * kGamma;
    const uint64_t zb = c.seedB + (g * s.words_per_group + wb + 1) * kGamma;
    PartyTriple t;
    if (p == 0) {
        t.a = mix64(za);
        t.b = mix64(zb);
        t.c = need_c ? mix64(zb + 2 * kGamma) : 0;
    } else {
        t.a = mix64(za + 1 * kGamma);
        t.b = mix64(zb + 1 * kGamma);
        t.c = 0;
        if (need_c) {   // the dealer's c_1 = ((a_0 ^ a_1) & (b_0 ^ b_1)) ^ c_0
            const uint64_t a0 = mix64(za), b0 = mix64(zb), c0 = mix64(zb + 2 * kGamma);
            t.c = ((a0 ^ t.a) & (b0 ^ t.b)) ^ c0;
        }
    }
    return t;
}

// Z_p = c_p ^ (d & b_p) ^ (e & a_p), party 0 also takes d & e.
__device__ __forceinline__ uint64_t party_and_finish(const PartyTriple &t, int p, uint64_t d, uint64_t e)
{
    uint64_t z = t.c ^ (d & t.b) ^ (e & t.a);
    if (p == 0) z ^= d & e;
    return z;
}

__device__ __forceinline__ uint64_t party_live(const PartyCtx &c, const PartyShape &s, uint64_t g)
{
    const uint64_t first = g * (uint64_t)s.L;
    const uint64_t cnt = c.n - first;
    if (cnt >= (uint64_t)s.L) return s.live;
    return (1ull << (cnt * (uint64_t)s.w)) - 1;     // cnt * w < 64 for a partial group
}

constexpr int kPartyBlock = 256;

// ---- "slice": load own shares, slice and pack, send the gate-0 maskings --------------------------------------
// grid (ceil(G / 256), 2); thread = (group, party)
__global__ void __launch_bounds__(kPartyBlock) party_slice_kernel(const PartyCtx c, const PartyShape s)
{
    const uint64_t g = (uint64_t)blockIdx.x * kPartyBlock + threadIdx.x;
    const int p = blockIdx.y;
    if (g >= c.groups) return;
    const uint64_t first = g * (uint64_t)s.L;
    const int cnt = (c.n - first >= (uint64_t)s.L) ? s.L : (int)(c.n - first);
    uint64_t u = 0;
    for (int j = 0; j < cnt; ++j) u |= ((c.x[p][first + j] >> s.k) & s.field) << (j * s.w);
    c.S[p][g] = u;                       // S_p = P_p = X_p ^ Y_p: party p's own slice, the other operand's share is 0
    c.P[p][g] = u;
    // gate 0 = X AND Y with X = (u_0, 0), Y = (0, u_1)
    const PartyTriple t = party_triple(c, s, p, g, 0, false);
    const uint64_t live = party_live(c, s, g);
    c.wire[p][2 * g + 0] = ((p == 0 ? u : 0) ^ t.a) & live;
    c.wire[p][2 * g + 1] = ((p == 1 ? u : 0) ^ t.b) & live;
}

// ---- prefix round r: finish the gates opened in the previous message, send this round's four maskings --------
__global__ void __launch_bounds__(kPartyBlock) party_round_kernel(const PartyCtx c, const PartyShape s, const int r)
{
    const uint64_t g = (uint64_t)blockIdx.x * kPartyBlock + threadIdx.x;
    const int p = blockIdx.y;
    if (g >= c.groups) return;
    uint64_t P = c.P[p][g], G;
    if (r == 0) {
        const uint64_t d = c.wire[0][2 * g] ^ c.wire[1][2 * g], e = c.wire[0][2 * g + 1] ^ c.wire[1][2 * g + 1];
        G = party_and_finish(party_triple(c, s, p, g, 0, true), p, d, e);
    } else {
        const uint64_t pr = (uint64_t)s.per_round;
        const uint64_t *w0 = c.wire[0] + 2 * c.groups + pr * c.groups * (uint64_t)(r - 1) + pr * g;
        const uint64_t *w1 = c.wire[1] + 2 * c.groups + pr * c.groups * (uint64_t)(r - 1) + pr * g;
        // opened values of the previous round: d, e of its G-update, then d, e of its P-update (d is shared on
        // the shared-mask layout)
        const uint64_t dT = w0[0] ^ w1[0], eT = w0[1] ^ w1[1];
        const uint64_t dP = s.shared ? dT : (w0[2] ^ w1[2]), eP = s.shared ? (w0[2] ^ w1[2]) : (w0[3] ^ w1[3]);
        const uint64_t T = party_and_finish(party_triple(c, s, p, g, 1 + 2 * (r - 1), true), p, dT, eT);
        const uint64_t Pn = party_and_finish(party_triple(c, s, p, g, 2 + 2 * (r - 1), true), p, dP, eP);
        G = c.G[p][g] ^ T;
        P = Pn;
    }
    c.G[p][g] = G;
    c.P[p][g] = P;
    const int sh = 1 << r;
    const uint64_t keep = s.keep[r], live = party_live(c, s, g);
    const PartyTriple tT = party_triple(c, s, p, g, 1 + 2 * r, false);
    const PartyTriple tP = party_triple(c, s, p, g, 2 + 2 * r, false);
    uint64_t *out = c.wire[p] + 2 * c.groups + (uint64_t)s.per_round * c.groups * (uint64_t)r + (uint64_t)s.per_round * g;
    out[0] = (P ^ tT.a) & live;
    out[1] = (((G << sh) & keep) ^ tT.b) & live;
    if (s.shared) {             // tP.a is the same word as tT.a: P ^ a has been sent already
        out[2] = (((P << sh) & keep) ^ tP.b) & live;
    } else {
        out[2] = (P ^ tP.a) & live;
        out[3] = (((P << sh) & keep) ^ tP.b) & live;
    }
}

// ---- "sign": finish the last G-update, take the sign share of every field, mask it with the dealer bit --------
__global__ void __launch_bounds__(kPartyBlock) party_sign_kernel(const PartyCtx c, const PartyShape s)
{
    const uint64_t g = (uint64_t)blockIdx.x * kPartyBlock + threadIdx.x;
    const int p = blockIdx.y;
    if (g >= c.groups) return;
    uint64_t G;
    if (s.R == 0) {
        const uint64_t d = c.wire[0][2 * g] ^ c.wire[1][2 * g], e = c.wire[0][2 * g + 1] ^ c.wire[1][2 * g + 1];
        G = party_and_finish(party_triple(c, s, p, g, 0, true), p, d, e);
    } else {
        const int r = s.R - 1;
        const uint64_t pr = (uint64_t)s.per_round;
        const uint64_t *w0 = c.wire[0] + 2 * c.groups + pr * c.groups * (uint64_t)r + pr * g;
        const uint64_t *w1 = c.wire[1] + 2 * c.groups + pr * c.groups * (uint64_t)r + pr * g;
        G = c.G[p][g] ^ party_and_finish(party_triple(c, s, p, g, 1 + 2 * r, true), p, w0[0] ^ w1[0], w0[1] ^ w1[1]);
    }
    const uint64_t sum = c.S[p][g] ^ ((G << 1) & s.keep1);
    const uint64_t wb = mix64(c.seedB + (g * s.words_per_group + s.words_per_group) * kGamma);   // the group's last word
    const uint64_t first = g * (uint64_t)s.L;
    const int cnt = (c.n - first >= (uint64_t)s.L) ? s.L : (int)(c.n - first);
    uint64_t zb = 0;
    for (int j = 0; j < cnt; ++j) {
        const uint64_t sign = (sum >> (j * s.w + s.w - 1)) & 1;
        const uint64_t rho = (wb >> (2 * j + p)) & 1;
        zb |= (sign ^ rho) << j;
    }
    c.Z[p][g] = zb;
}

// ---- B2A message: pack one bit per element, 64 elements per word ------------------------------------------------
__global__ void __launch_bounds__(kPartyBlock) party_b2a_kernel(const PartyCtx c, const PartyShape s)
{
    const uint64_t t = (uint64_t)blockIdx.x * kPartyBlock + threadIdx.x;
    const int p = blockIdx.y;
    const uint64_t words = (c.n + 63) / 64;
    if (t >= words) return;
    const uint64_t first = 64 * t;
    const int cnt = (c.n - first >= 64) ? 64 : (int)(c.n - first);
    uint64_t g = first / (uint64_t)s.L;
    int j = (int)(first - g * (uint64_t)s.L);
    uint64_t zb = c.Z[p][g], word = 0;
    for (int b = 0; b < cnt; ++b) {
        word |= ((zb >> j) & 1) << b;
        if (++j == s.L && b + 1 < cnt) {
            j = 0;
            zb = c.Z[p][++g];
        }
    }
    c.wire[p][c.off_b2a + t] = word;
}

// ---- multiply openings: read the opened B2A bit, form the DReLU share, send x_p - a_p and DReLU_p - b_p ---------
__global__ void __launch_bounds__(kPartyBlock) party_mul_send_kernel(const PartyCtx c, const PartyShape s)
{
    const uint64_t i = (uint64_t)blockIdx.x * kPartyBlock + threadIdx.x;
    const int p = blockIdx.y;
    if (i >= c.n) return;
    const uint64_t z = ((c.wire[0][c.off_b2a + i / 64] ^ c.wire[1][c.off_b2a + i / 64]) >> (i % 64)) & 1;
    const uint64_t zA = c.seedA + (6 * i + 1) * kGamma;
    const uint64_t rA0 = mix64(zA);
    uint64_t D;
    if (p == 0) {
        const uint64_t beta = z ? (1 - rA0) : rA0;          // beta_0 = r^A_0 + z - 2 z r^A_0
        D = 1 - beta;
    } else {
        // the dealer's arithmetic share of its bit for party 1: r - r^A_0
        const uint64_t g = i / (uint64_t)s.L;
        const int j = (int)(i - g * (uint64_t)s.L);
        const uint64_t wb = mix64(c.seedB + (g * s.words_per_group + s.words_per_group) * kGamma);
        const uint64_t r = ((wb >> (2 * j)) ^ (wb >> (2 * j + 1))) & 1;
        const uint64_t rA1 = r - rA0;
        const uint64_t beta = z ? (0 - rA1) : rA1;          // beta_1 = r^A_1 - 2 z r^A_1
        D = 0 - beta;
    }
    c.D[p][i] = D;
    const uint64_t a = mix64(zA + (uint64_t)(1 + p) * kGamma);      // A[6i+1] / A[6i+2]
    const uint64_t b = mix64(zA + (uint64_t)(3 + p) * kGamma);      // A[6i+3] / A[6i+4]
    c.wire[p][c.off_mul + 2 * i + 0] = c.x[p][i] - a;
    c.wire[p][c.off_mul + 2 * i + 1] = D - b;
}

// ---- result: ReLU_p = c_p + eps b_p + delta a_p (+ eps delta for party 0) ---------------------------------------
__global__ void __launch_bounds__(kPartyBlock) party_mul_finish_kernel(const PartyCtx c, const PartyShape s)
{
    const uint64_t i = (uint64_t)blockIdx.x * kPartyBlock + threadIdx.x;
    const int p = blockIdx.y;
    if (i >= c.n) return;
    (void)s;
    const uint64_t eps = c.wire[0][c.off_mul + 2 * i] + c.wire[1][c.off_mul + 2 * i];
    const uint64_t del = c.wire[0][c.off_mul + 2 * i + 1] + c.wire[1][c.off_mul + 2 * i + 1];
    const uint64_t zA = c.seedA + (6 * i + 1) * kGamma;
    const uint64_t a0 = mix64(zA + 1 * kGamma), b0 = mix64(zA + 3 * kGamma), c0 = mix64(zA + 5 * kGamma);
    uint64_t out;
    if (p == 0) {
        out = c0 + eps * b0 + del * a0 + eps * del;
    } else {
        const uint64_t a1 = mix64(zA + 2 * kGamma), b1 = mix64(zA + 4 * kGamma);
        const uint64_t c1 = (a0 + a1) * (b0 + b1) - c0;             // the dealer's share of c for party 1
        out = c1 + eps * b1 + del * a1;
    }
    c.out[p][i] = out;
}

}  // namespace hb
