/*
 * hb_ref.c -- CPU oracle for reduced-ring secret-shared DReLU / ReLU.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, per-element statement
 * of what the GPU library must compute.  Only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may use it; the product never calls it and shares
 * no code, header, table or constant generator with it.
 *
 * What it follows (paper = "Approximating ReLU on a Reduced Ring for Efficient
 * MPC-based Private Inference"):
 *   - notation x[hi:lo] and shares on Z_2^N ............ Sec. 2.2 "Notations"
 *   - ReLU = x * DReLU(x) ............................... Eq. 1, Eq. 2
 *   - A2B by an adder circuit on XOR shares, AND gates
 *     through Beaver triples, sign = MSB, B2A, 1 - sign . Sec. 2.2 "Evaluating ReLU with GMW"
 *   - DReLU evaluated on the slice of each share only ... Eq. 3, Sec. 3.1 (example, Thm 1, Thm 2)
 *   - depth ceil(log2 w) circuit, w-bit fields packed
 *     into 64-bit words ................................. Sec. 4.2
 *
 * The paper leaves the adder, the B2A construction, the triple source and the
 * party that adds public terms open.  The readings used here (Kogge-Stone with
 * zeros shifted in, one dealer bit for B2A, party 0 adds every public term,
 * SplitMix64 dealer streams with L = min(floor(64/w),32) fields per binary
 * word) are this project's protocol definition; the argument convention is
 * (k, m) = (lowest kept bit, one past the highest kept bit), w = m - k, i.e.
 * the paper's x[m:k].
 *
 * A second dealer layout ("variant 1") is offered beside the standard one: the
 * two AND gates of a prefix round both have the old propagate word P as first
 * operand, so one mask a serves both (P ^ a is opened once), and the round
 * opens 3w bits instead of 4w.  The circuit, and so every reconstructed
 * quantity, is unchanged; only the dealer words and the shares differ.
 *
 * Pins: every reconstructed quantity (adder sum, sign, DReLU, ReLU, opened-bit
 * counts, the generator) is pinned by the non-GPU tests against closed forms,
 * brute force on an 8-bit ring, the paper's worked example and published
 * generator vectors.  The VALUES OF THE INDIVIDUAL OUTPUT SHARES depend on the
 * dealer layout chosen by this project and are "parity unpinned" by the paper.
 *
 * Everything is integer; ring_bits (N) selects the arithmetic ring Z_2^N,
 * 1 <= N <= 64.  N = 64 is the production ring, N = 8 is used for brute force.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

#define HB_REF_OK 0
#define HB_REF_EINVAL (-1)

/* ------------------------------------------------------------------ */
/* Dealer randomness: SplitMix64 (public-domain generator).            */
/* ------------------------------------------------------------------ */

static const uint64_t GAMMA = 0x9E3779B97F4A7C15ULL;

uint64_t hb_ref_mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

/* One step of a SplitMix64 generator: advance the state, return the output. */
uint64_t hb_ref_sm_next(uint64_t *state)
{
    *state += GAMMA;
    return hb_ref_mix64(*state);
}

/* SM(s)[j]: the j-th (0-based) output of a generator whose state starts at s.
 * After j+1 steps the state is s + (j+1)*GAMMA, so the output can be indexed. */
uint64_t hb_ref_sm(uint64_t s, uint64_t j)
{
    return hb_ref_mix64(s + (j + 1) * GAMMA);
}

uint64_t hb_ref_tensor_seed(uint64_t root_seed, uint64_t tensor_id)
{
    return hb_ref_sm(root_seed, 2 + tensor_id);
}

/* ------------------------------------------------------------------ */
/* Shape of the protocol for one (k, m).                               */
/* ------------------------------------------------------------------ */

typedef struct {
    int k, m, w;        /* slice [k, m), width w                               */
    int R;              /* prefix rounds: 0 if w == 1 else ceil(log2 w)        */
    int L;              /* w-bit fields per 64-bit dealer word                 */
    uint64_t Wg;        /* dealer words per group of L elements                */
    uint64_t mask;      /* 2^w - 1                                             */
    uint64_t ring;      /* 2^N - 1                                             */
    uint64_t seedB;     /* binary-material stream   B[j] = SM(seedB)[j]        */
    uint64_t seedA;     /* arithmetic-material stream A[j] = SM(seedA)[j]      */
    int variant;        /* 0: every gate has its own triple; 1: the two gates of a round share the mask of P */
} shape_t;

static int rounds_for(int w)
{
    int R = 0;
    while ((1 << R) < w) R++;
    return R;
}

/* Position, inside a group's run of dealer words, of slot (0:a_0 1:a_1 2:b_0 3:b_1 4:c_0) of gate q.
 * Standard layout: five words per gate.  Shared-mask variant: gate 0 as before; round r owns eight words
 * a_0 a_1 | b_0 b_1 c_0 of the G-update | b_0 b_1 c_0 of the P-update, the mask a of P serving both gates. */
static uint64_t word_of(const shape_t *s, int q, int slot)
{
    if (!s->variant || q == 0) return 5u * (uint64_t)q + (uint64_t)slot;
    const int r = (q - 1) / 2, is_p_update = (q - 1) % 2;
    const uint64_t base = 5u + 8u * (uint64_t)r;
    if (slot < 2 || !is_p_update) return base + (uint64_t)slot;
    return base + 3u + (uint64_t)slot;
}

static uint64_t b2a_word_of(const shape_t *s)
{
    return s->variant ? 5u + 8u * (uint64_t)s->R : 5u * (uint64_t)(1 + 2 * s->R);
}

static int make_shape_v(shape_t *s, int k, int m, uint64_t seed, int ring_bits, int variant)
{
    if (variant != 0 && variant != 1) return HB_REF_EINVAL;
    s->variant = variant;
    if (ring_bits < 1 || ring_bits > 64) return HB_REF_EINVAL;
    if (k < 0 || m <= k || m > ring_bits) return HB_REF_EINVAL;
    s->k = k;
    s->m = m;
    s->w = m - k;
    s->R = rounds_for(s->w);
    s->L = 64 / s->w;
    if (s->L > 32) s->L = 32;
    s->Wg = b2a_word_of(s) + 1;
    s->mask = (s->w == 64) ? ~0ULL : ((1ULL << s->w) - 1);
    s->ring = (ring_bits == 64) ? ~0ULL : ((1ULL << ring_bits) - 1);
    s->seedB = hb_ref_sm(seed, 0);
    s->seedA = hb_ref_sm(seed, 1);
    return HB_REF_OK;
}

static int make_shape(shape_t *s, int k, int m, uint64_t seed, int ring_bits)
{
    return make_shape_v(s, k, m, seed, ring_bits, 0);
}

/* Opened (publicly reconstructed) bits: gate 0 opens 2w, every prefix round
 * opens 4w (two AND gates), B2A opens 1, the multiply opens two ring elements
 * (counted as 128 on the 64-bit production ring).
 * Variant 1: a prefix round opens P ^ a once, for both gates, and the two
 * second operands: 3w bits instead of 4w. */
uint64_t hb_ref_opened_bits_v(int relu, int k, int m, uint64_t n, int variant)
{
    if (k < 0 || m <= k || m > 64) return 0;
    uint64_t w = (uint64_t)(m - k);
    uint64_t R = (uint64_t)rounds_for((int)w);
    uint64_t per = (variant ? 2 * w + 3 * w * R : 2 * w * (1 + 2 * R)) + 1;
    if (relu) per += 128;
    return n * per;
}

uint64_t hb_ref_opened_bits(int relu, int k, int m, uint64_t n)
{
    return hb_ref_opened_bits_v(relu, k, m, n, 0);
}

/* ------------------------------------------------------------------ */
/* One AND gate on XOR shares through a Beaver triple.                  */
/* U is masked by a, V is masked by b; d and e are opened.              */
/* ------------------------------------------------------------------ */

void hb_ref_and_gate(uint64_t U0, uint64_t U1, uint64_t V0, uint64_t V1,
                     uint64_t a0, uint64_t a1, uint64_t b0, uint64_t b1,
                     uint64_t c0, uint64_t mask, uint64_t *Z0, uint64_t *Z1)
{
    uint64_t c1 = (((a0 ^ a1) & (b0 ^ b1)) ^ c0) & mask;
    uint64_t d = (U0 ^ a0 ^ U1 ^ a1) & mask;
    uint64_t e = (V0 ^ b0 ^ V1 ^ b1) & mask;
    *Z0 = (c0 ^ (d & b0) ^ (e & a0) ^ (d & e)) & mask;
    *Z1 = (c1 ^ (d & b1) ^ (e & a1)) & mask;
}

/* ------------------------------------------------------------------ */
/* One element, start to finish.                                        */
/* ------------------------------------------------------------------ */

typedef struct {
    uint64_t u[2];      /* sliced shares on Z_2^w                         */
    uint64_t sum[2];    /* XOR shares of (u0 + u1) mod 2^w, all w bits    */
    uint64_t sign[2];   /* XOR shares of the MSB of that sum              */
    uint64_t drelu[2];  /* arithmetic shares of 1 - sign on Z_2^N         */
    uint64_t relu[2];   /* arithmetic shares of x * (1 - sign) on Z_2^N   */
    /* what each party sends for every opening (its masked share), gate q = 0 .. 2R */
    uint64_t send_d[2][13], send_e[2][13];  /* U_p ^ a_p, V_p ^ b_p of gate q        */
    uint64_t send_z[2];                     /* sign_p ^ rho_p                         */
    uint64_t send_eps[2], send_del[2];      /* x_p - a_p, DReLU_p - b_p               */
} elem_t;

static void eval_element(const shape_t *s, uint64_t i, uint64_t x0, uint64_t x1,
                         int want_relu, elem_t *t)
{
    const uint64_t mask = s->mask, ring = s->ring;
    const int w = s->w;
    const uint64_t g = i / (uint64_t)s->L;        /* group                     */
    const unsigned j = (unsigned)(i % (uint64_t)s->L); /* field inside the group */
    const unsigned fsh = j * (unsigned)w;         /* field position in a word  */
    const uint64_t base = g * s->Wg;              /* first dealer word of group */
    int p, r;

    x0 &= ring;
    x1 &= ring;

    /* slice: logical shift of the two's-complement pattern, keep w bits */
    t->u[0] = (x0 >> s->k) & mask;
    t->u[1] = (x1 >> s->k) & mask;

    /* each party binary-shares its own slice: X = (u0, 0), Y = (0, u1) */
    uint64_t X[2] = { t->u[0], 0 };
    uint64_t Y[2] = { 0, t->u[1] };
    uint64_t P[2], S[2], G[2];

    for (p = 0; p < 2; p++) {
        P[p] = X[p] ^ Y[p];
        S[p] = P[p];
    }

#define FIELD(q, slot) ((hb_ref_sm(s->seedB, base + word_of(s, (q), (slot))) >> fsh) & mask)
#define AND_GATE(q, U, V, Z) \
    t->send_d[0][q] = ((U)[0] ^ FIELD(q, 0)) & mask; t->send_d[1][q] = ((U)[1] ^ FIELD(q, 1)) & mask; \
    t->send_e[0][q] = ((V)[0] ^ FIELD(q, 2)) & mask; t->send_e[1][q] = ((V)[1] ^ FIELD(q, 3)) & mask; \
    hb_ref_and_gate((U)[0], (U)[1], (V)[0], (V)[1], FIELD(q, 0), FIELD(q, 1), \
                    FIELD(q, 2), FIELD(q, 3), FIELD(q, 4), mask, &(Z)[0], &(Z)[1])

    /* gate 0: generate = X AND Y */
    AND_GATE(0, X, Y, G);

    /* Kogge-Stone prefix rounds, zeros shifted in, both gates use the old P */
    for (r = 0; r < s->R; r++) {
        const int sh = 1 << r;
        uint64_t Gs[2], Ps[2], T[2], Pn[2];
        for (p = 0; p < 2; p++) {
            Gs[p] = (G[p] << sh) & mask;
            Ps[p] = (P[p] << sh) & mask;
        }
        AND_GATE(1 + 2 * r, P, Gs, T);
        AND_GATE(2 + 2 * r, P, Ps, Pn);
        for (p = 0; p < 2; p++) {
            G[p] ^= T[p];
            P[p] = Pn[p];
        }
    }
#undef AND_GATE
#undef FIELD

    /* sum bit i = propagate_i XOR carry into i; carry into i = G[i-1] */
    for (p = 0; p < 2; p++) {
        t->sum[p] = S[p] ^ ((G[p] << 1) & mask);
        t->sign[p] = (t->sum[p] >> (w - 1)) & 1;
    }

    /* B2A with one dealer bit r = rho0 ^ rho1, shared both ways */
    const uint64_t Wb = hb_ref_sm(s->seedB, base + b2a_word_of(s));
    const uint64_t rho0 = (Wb >> (2 * j)) & 1;
    const uint64_t rho1 = (Wb >> (2 * j + 1)) & 1;
    const uint64_t rbit = rho0 ^ rho1;
    const uint64_t z = t->sign[0] ^ rho0 ^ t->sign[1] ^ rho1;    /* opened */
    t->send_z[0] = t->sign[0] ^ rho0;
    t->send_z[1] = t->sign[1] ^ rho1;
    uint64_t rA[2], beta[2];
    rA[0] = hb_ref_sm(s->seedA, 6 * i) & ring;
    rA[1] = (rbit - rA[0]) & ring;
    /* sign = z XOR r = z + r - 2 z r ; party 0 adds the public z */
    beta[0] = (rA[0] + z - 2 * z * rA[0]) & ring;
    beta[1] = (rA[1] - 2 * z * rA[1]) & ring;
    t->drelu[0] = (1 - beta[0]) & ring;
    t->drelu[1] = (0 - beta[1]) & ring;

    t->relu[0] = t->relu[1] = 0;
    t->send_eps[0] = t->send_eps[1] = t->send_del[0] = t->send_del[1] = 0;
    if (!want_relu) return;

    /* Beaver multiply x * DReLU on Z_2^N */
    const uint64_t a0 = hb_ref_sm(s->seedA, 6 * i + 1) & ring;
    const uint64_t a1 = hb_ref_sm(s->seedA, 6 * i + 2) & ring;
    const uint64_t b0 = hb_ref_sm(s->seedA, 6 * i + 3) & ring;
    const uint64_t b1 = hb_ref_sm(s->seedA, 6 * i + 4) & ring;
    const uint64_t c0 = hb_ref_sm(s->seedA, 6 * i + 5) & ring;
    const uint64_t c1 = ((a0 + a1) * (b0 + b1) - c0) & ring;
    const uint64_t eps = ((x0 - a0) + (x1 - a1)) & ring;                       /* opened */
    const uint64_t del = ((t->drelu[0] - b0) + (t->drelu[1] - b1)) & ring;     /* opened */
    t->send_eps[0] = (x0 - a0) & ring;
    t->send_eps[1] = (x1 - a1) & ring;
    t->send_del[0] = (t->drelu[0] - b0) & ring;
    t->send_del[1] = (t->drelu[1] - b1) & ring;
    t->relu[0] = (c0 + eps * b0 + del * a0 + eps * del) & ring;
    t->relu[1] = (c1 + eps * b1 + del * a1) & ring;
}

/* ------------------------------------------------------------------ */
/* Array entry points (host pointers).                                  */
/* ------------------------------------------------------------------ */

/* Elements first .. first+n-1 of a tensor; share0/share1/out0/out1 point at
 * element `first`.  what: 0 = DReLU shares, 1 = ReLU shares,
 * 2 = XOR shares of the full w-bit adder sum, 3 = XOR shares of the sign bit,
 * 4 = the sliced shares u0, u1.
 * variant: 0 = one triple per gate; 1 = the two gates of a prefix round share the mask of P. */
int hb_ref_eval_range_v(const int64_t *share0, const int64_t *share1, uint64_t first, uint64_t n,
                        int k, int m, uint64_t seed, int ring_bits, int variant, int what,
                        int64_t *out0, int64_t *out1)
{
    shape_t s;
    uint64_t i;
    if (what < 0 || what > 4) return HB_REF_EINVAL;
    if (make_shape_v(&s, k, m, seed, ring_bits, variant) != HB_REF_OK) return HB_REF_EINVAL;
    if (n > 0 && (!share0 || !share1 || !out0 || !out1)) return HB_REF_EINVAL;
    for (i = 0; i < n; i++) {
        elem_t t;
        eval_element(&s, first + i, (uint64_t)share0[i], (uint64_t)share1[i], what == 1, &t);
        const uint64_t *src = what == 0 ? t.drelu : what == 1 ? t.relu : what == 2 ? t.sum
                              : what == 3 ? t.sign : t.u;
        out0[i] = (int64_t)src[0];
        out1[i] = (int64_t)src[1];
    }
    return HB_REF_OK;
}

int hb_ref_eval_range(const int64_t *share0, const int64_t *share1, uint64_t first, uint64_t n,
                      int k, int m, uint64_t seed, int ring_bits, int what,
                      int64_t *out0, int64_t *out1)
{
    return hb_ref_eval_range_v(share0, share1, first, n, k, m, seed, ring_bits, 0, what, out0, out1);
}

/* Scattered elements: element index[i] of the tensor carries the share values
 * share0[i], share1[i].  Same `what` codes as above. */
int hb_ref_eval_at_v(const int64_t *share0, const int64_t *share1, const uint64_t *index, uint64_t count,
                     int k, int m, uint64_t seed, int ring_bits, int variant, int what,
                     int64_t *out0, int64_t *out1)
{
    shape_t s;
    uint64_t i;
    if (what < 0 || what > 4) return HB_REF_EINVAL;
    if (make_shape_v(&s, k, m, seed, ring_bits, variant) != HB_REF_OK) return HB_REF_EINVAL;
    if (count > 0 && (!share0 || !share1 || !index || !out0 || !out1)) return HB_REF_EINVAL;
    for (i = 0; i < count; i++) {
        elem_t t;
        eval_element(&s, index[i], (uint64_t)share0[i], (uint64_t)share1[i], what == 1, &t);
        const uint64_t *src = what == 0 ? t.drelu : what == 1 ? t.relu : what == 2 ? t.sum
                              : what == 3 ? t.sign : t.u;
        out0[i] = (int64_t)src[0];
        out1[i] = (int64_t)src[1];
    }
    return HB_REF_OK;
}

int hb_ref_eval_at(const int64_t *share0, const int64_t *share1, const uint64_t *index, uint64_t count,
                   int k, int m, uint64_t seed, int ring_bits, int what,
                   int64_t *out0, int64_t *out1)
{
    return hb_ref_eval_at_v(share0, share1, index, count, k, m, seed, ring_bits, 0, what, out0, out1);
}

int hb_ref_drelu(const int64_t *share0, const int64_t *share1, uint64_t n, int k, int m,
                 uint64_t seed, int ring_bits, int64_t *out0, int64_t *out1, uint64_t *opened_bits)
{
    int st = hb_ref_eval_range(share0, share1, 0, n, k, m, seed, ring_bits, 0, out0, out1);
    if (st == HB_REF_OK && opened_bits) *opened_bits = hb_ref_opened_bits(0, k, m, n);
    return st;
}

int hb_ref_relu(const int64_t *share0, const int64_t *share1, uint64_t n, int k, int m,
                uint64_t seed, int ring_bits, int64_t *out0, int64_t *out1, uint64_t *opened_bits)
{
    int st = hb_ref_eval_range(share0, share1, 0, n, k, m, seed, ring_bits, 1, out0, out1);
    if (st == HB_REF_OK && opened_bits) *opened_bits = hb_ref_opened_bits(1, k, m, n);
    return st;
}

/* Reconstruction: sum of the shares mod 2^N, or their XOR. */
int hb_ref_open(const int64_t *share0, const int64_t *share1, uint64_t n, int binary,
                int ring_bits, int64_t *out)
{
    uint64_t i, ring;
    if (ring_bits < 1 || ring_bits > 64) return HB_REF_EINVAL;
    if (n > 0 && (!share0 || !share1 || !out)) return HB_REF_EINVAL;
    ring = (ring_bits == 64) ? ~0ULL : ((1ULL << ring_bits) - 1);
    for (i = 0; i < n; i++) {
        uint64_t a = (uint64_t)share0[i], b = (uint64_t)share1[i];
        out[i] = (int64_t)((binary ? (a ^ b) : (a + b)) & ring);
    }
    return HB_REF_OK;
}

/* ------------------------------------------------------------------ */
/* Zero-error search for the high cut ("eco" strategy, Sec. 4.1.2):     */
/* evaluate DReLU on [0, m) for every m and see whether the result      */
/* differs from the full ring.  counts[m-1] = number of elements whose  */
/* reconstructed DReLU at (0, m) differs from the one at (0, N).        */
/* ------------------------------------------------------------------ */
int hb_ref_eco_scan(const int64_t *share0, const int64_t *share1, uint64_t n, uint64_t seed, int ring_bits,
                    uint64_t *counts)
{
    shape_t full, cut;
    uint64_t i;
    int m;
    if (!counts || make_shape(&full, 0, ring_bits, seed, ring_bits) != HB_REF_OK) return HB_REF_EINVAL;
    if (n > 0 && (!share0 || !share1)) return HB_REF_EINVAL;
    for (m = 1; m <= 64; m++) counts[m - 1] = 0;
    for (m = 1; m <= ring_bits; m++) {
        if (make_shape(&cut, 0, m, seed, ring_bits) != HB_REF_OK) return HB_REF_EINVAL;
        for (i = 0; i < n; i++) {
            elem_t a, b;
            eval_element(&full, i, (uint64_t)share0[i], (uint64_t)share1[i], 0, &a);
            eval_element(&cut, i, (uint64_t)share0[i], (uint64_t)share1[i], 0, &b);
            if (((a.drelu[0] + a.drelu[1]) & full.ring) != ((b.drelu[0] + b.drelu[1]) & full.ring)) counts[m - 1]++;
        }
    }
    return HB_REF_OK;
}

/* The zero-error choice: the smallest m such that no m' >= m shows a mismatch. */
int hb_ref_eco_choose(const uint64_t *counts, int ring_bits)
{
    int m = ring_bits;
    while (m > 1 && counts[m - 2] == 0) m--;
    return m;
}

/* ------------------------------------------------------------------ */
/* What the two parties would put on the wire for one ReLU (Sec. 2.2:   */
/* every AND, the B2A and the multiply open masked values; Sec. 4.2:    */
/* the w-bit fields travel packed in 64-bit words).  Party p's wire is  */
/* an array of 64-bit words in sections:                                */
/*   gate 0      : 2 words per group  [2g + 0] = U_p^a_p, [2g + 1] = V_p^b_p            */
/*   round r     : 4 words per group  [4g + 0,1] = G-update gate, [4g + 2,3] = P-update  */
/*   B2A         : ceil(n/64) words, bit i%64 of word i/64 = sign_p ^ rho_p of element i */
/*   multiply    : 2 words per element [2i] = x_p - a_p, [2i + 1] = DReLU_p - b_p        */
/* Field j of a group word sits at bit j*w; bits of no element are 0.   */
/* ------------------------------------------------------------------ */
/* Variant 1 (one mask of P per round): a round sends three words per group instead of four,           */
/*   round r     : 3 words per group  [3g + 0] = P_p^a_p (serves both gates), [3g + 1] = (G<<s)_p^b_p   */
/*                 of the G-update, [3g + 2] = (P<<s)_p^b'_p of the P-update.                           */
uint64_t hb_ref_wire_words_v(uint64_t n, int k, int m, int variant)
{
    shape_t s;
    if (make_shape_v(&s, k, m, 0, 64, variant) != HB_REF_OK) return 0;
    const uint64_t G = (n + (uint64_t)s.L - 1) / (uint64_t)s.L;
    const uint64_t per_round = variant ? 3 : 4;
    return 2 * G + per_round * G * (uint64_t)s.R + (n + 63) / 64 + 2 * n;
}

uint64_t hb_ref_wire_words(uint64_t n, int k, int m)
{
    return hb_ref_wire_words_v(n, k, m, 0);
}

int hb_ref_relu_wire_v(const int64_t *share0, const int64_t *share1, uint64_t n, int k, int m, uint64_t seed,
                       int variant, uint64_t *wire0, uint64_t *wire1)
{
    shape_t s;
    uint64_t i, words;
    int p, r;
    if (make_shape_v(&s, k, m, seed, 64, variant) != HB_REF_OK) return HB_REF_EINVAL;
    if (n > 0 && (!share0 || !share1 || !wire0 || !wire1)) return HB_REF_EINVAL;
    words = hb_ref_wire_words_v(n, k, m, variant);
    for (i = 0; i < words; i++) wire0[i] = wire1[i] = 0;
    const uint64_t G = (n + (uint64_t)s.L - 1) / (uint64_t)s.L;
    const uint64_t per_round = variant ? 3 : 4;
    const uint64_t off_b2a = 2 * G + per_round * G * (uint64_t)s.R, off_mul = off_b2a + (n + 63) / 64;
    for (i = 0; i < n; i++) {
        elem_t t;
        uint64_t *wire[2] = { wire0, wire1 };
        const uint64_t g = i / (uint64_t)s.L;
        const unsigned sh = (unsigned)(i % (uint64_t)s.L) * (unsigned)s.w;
        eval_element(&s, i, (uint64_t)share0[i], (uint64_t)share1[i], 1, &t);
        for (p = 0; p < 2; p++) {
            wire[p][2 * g + 0] |= t.send_d[p][0] << sh;
            wire[p][2 * g + 1] |= t.send_e[p][0] << sh;
            for (r = 0; r < s.R; r++) {
                uint64_t *sec = wire[p] + 2 * G + per_round * G * (uint64_t)r;
                if (variant) {
                    /* the masked P is the same message for both gates of the round: sent once */
                    sec[3 * g + 0] |= t.send_d[p][1 + 2 * r] << sh;
                    sec[3 * g + 1] |= t.send_e[p][1 + 2 * r] << sh;
                    sec[3 * g + 2] |= t.send_e[p][2 + 2 * r] << sh;
                } else {
                    sec[4 * g + 0] |= t.send_d[p][1 + 2 * r] << sh;
                    sec[4 * g + 1] |= t.send_e[p][1 + 2 * r] << sh;
                    sec[4 * g + 2] |= t.send_d[p][2 + 2 * r] << sh;
                    sec[4 * g + 3] |= t.send_e[p][2 + 2 * r] << sh;
                }
            }
            wire[p][off_b2a + i / 64] |= t.send_z[p] << (i % 64);
            wire[p][off_mul + 2 * i + 0] = t.send_eps[p];
            wire[p][off_mul + 2 * i + 1] = t.send_del[p];
        }
    }
    return HB_REF_OK;
}

int hb_ref_relu_wire(const int64_t *share0, const int64_t *share1, uint64_t n, int k, int m, uint64_t seed,
                     uint64_t *wire0, uint64_t *wire1)
{
    return hb_ref_relu_wire_v(share0, share1, n, k, m, seed, 0, wire0, wire1);
}

/* ------------------------------------------------------------------ */
/* Float boundary of the simulator (Sec. 4.1.1; fixed point of          */
/* Sec. 2.2 / Sec. 3.1: x = round(2^16 x_f), ties to even).  NaN        */
/* encodes as 0; |2^16 x_f| is clamped to 2^62.                         */
/* ------------------------------------------------------------------ */
int64_t hb_ref_encode_f32(float v)
{
    double d = (double)v * 65536.0;
    if (isnan(d)) d = 0.0;
    if (d > 4611686018427387904.0) d = 4611686018427387904.0;
    if (d < -4611686018427387904.0) d = -4611686018427387904.0;
    return (int64_t)llrint(d);          /* default rounding mode: to nearest, ties to even */
}

float hb_ref_decode_f32(int64_t v)
{
    return (float)((double)v / 65536.0);
}

int hb_ref_share_f32(const float *x, uint64_t n, uint64_t share_seed, int64_t *share0, int64_t *share1)
{
    uint64_t i, state = share_seed;
    if (n > 0 && (!x || !share0 || !share1)) return HB_REF_EINVAL;
    for (i = 0; i < n; i++) {
        const uint64_t r = hb_ref_sm_next(&state);           /* step the generator: output i */
        share0[i] = (int64_t)r;
        share1[i] = (int64_t)((uint64_t)hb_ref_encode_f32(x[i]) - r);
    }
    return HB_REF_OK;
}

int hb_ref_reveal_f32(const int64_t *share0, const int64_t *share1, uint64_t n, float *y)
{
    uint64_t i;
    if (n > 0 && (!share0 || !share1 || !y)) return HB_REF_EINVAL;
    for (i = 0; i < n; i++) y[i] = hb_ref_decode_f32((int64_t)((uint64_t)share0[i] + (uint64_t)share1[i]));
    return HB_REF_OK;
}
