/*
 * hb_ref_mp.c -- CPU oracle for the reduced-ring DReLU / ReLU among p >= 2 parties.
 *
 * TEST INFRASTRUCTURE ONLY (see hb_ref.c).  Plain, slow, one element at a time.
 *
 * What it follows: the paper's setting allows any number of parties p >= 2
 * (Sec. 2.2 "Operation of CrypTen": a secret is split into p arithmetic shares;
 * Sec. 3.1.2 notes that the two-party analysis extends to more parties).  The
 * ReLU protocol is the one of Sec. 2.2 "Evaluating ReLU with GMW" with Eq. 3's
 * slicing: every party slices its own share, the p sliced shares are added on
 * XOR shares by adder circuits, sign = MSB, B2A, 1 - sign, Beaver multiply.
 *
 * The paper does not say how p > 2 binary numbers are added, nor how triples
 * are shared among p parties.  Readings used here (this project's protocol
 * definition; with p = 2 everything below is exactly hb_ref.c's protocol):
 *   - party q XOR-shares its slice trivially (its own share is the slice, the
 *     others' shares are zero);
 *   - the p shared numbers are summed by a tree of two-operand adders: level by
 *     level, neighbours (0,1), (2,3), ... are added and an odd last one is
 *     carried up; adders are numbered in the order they are evaluated;
 *   - every adder is the Kogge-Stone circuit of hb_ref.c (gate 0, R rounds of
 *     two AND gates on the old P, zeros shifted in); sum = S ^ (G << 1);
 *   - an AND gate among p parties uses a triple shared p ways: dealer words
 *     a_0..a_{p-1}, b_0..b_{p-1}, c_0..c_{p-2} (3p-1 words); c_{p-1} completes
 *     c = a & b; d = XOR_q (U_q ^ a_q), e = XOR_q (V_q ^ b_q) are opened;
 *     Z_q = c_q ^ (d & b_q) ^ (e & a_q) ^ [q = 0](d & e);
 *   - group g owns Wg = (p-1)(1+2R)(3p-1) + 1 binary words; gate t of adder s
 *     starts at word (s(1+2R) + t)(3p-1); the last word holds the B2A bits:
 *     bit p*j + q is rho_q of lane j, so L = min(floor(64/w), floor(64/p));
 *   - element i owns 4p-2 arithmetic words: rA_0..rA_{p-2} | a_0..a_{p-1} |
 *     b_0..b_{p-1} | c_0..c_{p-2}; rA_{p-1} = r - sum of the others (r = XOR of
 *     the rho bits); c_{p-1} = (sum a)(sum b) - sum of the other c;
 *   - party 0 adds every public term.
 *
 * Opened bits are counted per link and direction (what one party sends to one
 * other party): n * ((p-1) * 2w(1+2R) + 1 [+ 128]).
 *
 * Pins (non-GPU tests): p = 2 reproduces hb_ref.c share for share; for every p
 * the reconstructed adder sum equals (sum of the slices) mod 2^w, the full
 * ring is exact, the reconstructed ReLU equals x * DReLU, and a small ring is
 * checked by brute force over every share triple.  The values of the
 * individual output shares for p > 2 are "parity unpinned" by the paper.
 */
#include <stddef.h>
#include <stdint.h>

#define HB_REF_OK 0
#define HB_REF_EINVAL (-1)
#define HB_REF_MAX_PARTIES 8

uint64_t hb_ref_sm(uint64_t s, uint64_t j);     /* hb_ref.c: output j of the generator started at s */

typedef struct {
    int p, k, m, w, R, L, N;
    uint64_t mask, ring, Wg, gate_words, arith_words, seedB, seedA;
} mp_shape_t;

static int mp_rounds(int w)
{
    int r = 0;
    while ((1 << r) < w) r++;
    return r;
}

static int mp_make_shape(mp_shape_t *s, int parties, int k, int m, uint64_t seed, int ring_bits)
{
    if (parties < 2 || parties > HB_REF_MAX_PARTIES) return HB_REF_EINVAL;
    if (ring_bits < 1 || ring_bits > 64) return HB_REF_EINVAL;
    if (k < 0 || m <= k || m > ring_bits) return HB_REF_EINVAL;
    s->p = parties;
    s->k = k;
    s->m = m;
    s->N = ring_bits;
    s->w = m - k;
    s->R = mp_rounds(s->w);
    s->L = 64 / s->w < 64 / parties ? 64 / s->w : 64 / parties;
    s->mask = s->w == 64 ? ~0ULL : (1ULL << s->w) - 1;
    s->ring = ring_bits == 64 ? ~0ULL : (1ULL << ring_bits) - 1;
    s->gate_words = (uint64_t)(3 * parties - 1);
    s->Wg = (uint64_t)(parties - 1) * (uint64_t)(1 + 2 * s->R) * s->gate_words + 1;
    s->arith_words = (uint64_t)(4 * parties - 2);
    s->seedB = hb_ref_sm(seed, 0);
    s->seedA = hb_ref_sm(seed, 1);
    return HB_REF_OK;
}

uint64_t hb_ref_mp_opened_bits(int relu, int parties, int k, int m, uint64_t n)
{
    if (parties < 2 || parties > HB_REF_MAX_PARTIES || k < 0 || m <= k || m > 64) return 0;
    const uint64_t w = (uint64_t)(m - k), R = (uint64_t)mp_rounds((int)w);
    return n * ((uint64_t)(parties - 1) * 2 * w * (1 + 2 * R) + 1 + (relu ? 128 : 0));
}

typedef struct {
    uint64_t v[HB_REF_MAX_PARTIES];
} mp_val_t;

/* AND of two XOR-shared w-bit values; the gate's first dealer word is `word` of group `g`, this element's
 * field sits at bit `fsh` of every word. */
static mp_val_t mp_and(const mp_shape_t *s, uint64_t g, uint64_t word, unsigned fsh, const mp_val_t *U, const mp_val_t *V)
{
    const int p = s->p;
    uint64_t a[HB_REF_MAX_PARTIES], b[HB_REF_MAX_PARTIES], c[HB_REF_MAX_PARTIES];
    uint64_t as = 0, bs = 0, cs = 0, d = 0, e = 0;
    mp_val_t Z = {{0}};
    int q;
    for (q = 0; q < p; q++) {
        a[q] = (hb_ref_sm(s->seedB, g * s->Wg + word + (uint64_t)q) >> fsh) & s->mask;
        b[q] = (hb_ref_sm(s->seedB, g * s->Wg + word + (uint64_t)(p + q)) >> fsh) & s->mask;
        as ^= a[q];
        bs ^= b[q];
    }
    for (q = 0; q < p - 1; q++) {
        c[q] = (hb_ref_sm(s->seedB, g * s->Wg + word + (uint64_t)(2 * p + q)) >> fsh) & s->mask;
        cs ^= c[q];
    }
    c[p - 1] = (as & bs) ^ cs;                       /* the dealer completes c = a & b */
    for (q = 0; q < p; q++) {                        /* every party publishes U_q ^ a_q and V_q ^ b_q */
        d ^= U->v[q] ^ a[q];
        e ^= V->v[q] ^ b[q];
    }
    for (q = 0; q < p; q++) Z.v[q] = (c[q] ^ (d & b[q]) ^ (e & a[q])) & s->mask;
    Z.v[0] ^= d & e;
    return Z;
}

/* X + Y mod 2^w on XOR shares: adder number `adder` of the group. */
static mp_val_t mp_add(const mp_shape_t *s, uint64_t g, int adder, unsigned fsh, const mp_val_t *X, const mp_val_t *Y)
{
    const int p = s->p;
    const uint64_t first = (uint64_t)adder * (uint64_t)(1 + 2 * s->R) * s->gate_words;
    mp_val_t P, S, G, out;
    int q, r;
    for (q = 0; q < HB_REF_MAX_PARTIES; q++) P.v[q] = S.v[q] = out.v[q] = 0;
    for (q = 0; q < p; q++) P.v[q] = S.v[q] = X->v[q] ^ Y->v[q];
    G = mp_and(s, g, first, fsh, X, Y);
    for (r = 0; r < s->R; r++) {
        const int sh = 1 << r;
        mp_val_t Gs, Ps, T, Pn;
        for (q = 0; q < HB_REF_MAX_PARTIES; q++) Gs.v[q] = Ps.v[q] = 0;
        for (q = 0; q < p; q++) {
            Gs.v[q] = (G.v[q] << sh) & s->mask;
            Ps.v[q] = (P.v[q] << sh) & s->mask;
        }
        T = mp_and(s, g, first + (uint64_t)(1 + 2 * r) * s->gate_words, fsh, &P, &Gs);
        Pn = mp_and(s, g, first + (uint64_t)(2 + 2 * r) * s->gate_words, fsh, &P, &Ps);
        for (q = 0; q < p; q++) {
            G.v[q] ^= T.v[q];
            P.v[q] = Pn.v[q];
        }
    }
    for (q = 0; q < p; q++) out.v[q] = S.v[q] ^ ((G.v[q] << 1) & s->mask);
    return out;
}

typedef struct {
    uint64_t u[HB_REF_MAX_PARTIES], sum[HB_REF_MAX_PARTIES], sign[HB_REF_MAX_PARTIES];
    uint64_t drelu[HB_REF_MAX_PARTIES], relu[HB_REF_MAX_PARTIES];
} mp_elem_t;

static void mp_eval_element(const mp_shape_t *s, uint64_t i, const uint64_t *x_in, int want_relu, mp_elem_t *t)
{
    const int p = s->p;
    const uint64_t g = i / (uint64_t)s->L;
    const unsigned j = (unsigned)(i % (uint64_t)s->L);
    const unsigned fsh = j * (unsigned)s->w;
    uint64_t x[HB_REF_MAX_PARTIES];
    mp_val_t T[HB_REF_MAX_PARTIES];
    int q, t2, count, adder = 0;

    for (q = 0; q < p; q++) {
        x[q] = x_in[q] & s->ring;
        t->u[q] = (x[q] >> s->k) & s->mask;
    }
    /* party q shares its slice trivially */
    for (q = 0; q < p; q++) {
        for (t2 = 0; t2 < HB_REF_MAX_PARTIES; t2++) T[q].v[t2] = 0;
        T[q].v[q] = t->u[q];
    }
    /* tree of adders */
    count = p;
    while (count > 1) {
        int o = 0, a;
        for (a = 0; a + 1 < count; a += 2) {
            const mp_val_t sum = mp_add(s, g, adder++, fsh, &T[a], &T[a + 1]);
            T[o++] = sum;
        }
        if (count & 1) T[o++] = T[count - 1];
        count = o;
    }
    for (q = 0; q < p; q++) {
        t->sum[q] = T[0].v[q];
        t->sign[q] = (T[0].v[q] >> (s->w - 1)) & 1;
    }

    /* B2A of the sign with one dealer bit r = XOR of rho_q; DReLU = 1 - sign */
    const uint64_t Wb = hb_ref_sm(s->seedB, g * s->Wg + (s->Wg - 1));
    uint64_t z = 0, rbit = 0, rsum = 0, rA[HB_REF_MAX_PARTIES];
    for (q = 0; q < p; q++) {
        const uint64_t rho = (Wb >> ((unsigned)p * j + (unsigned)q)) & 1;
        z ^= t->sign[q] ^ rho;                               /* opened */
        rbit ^= rho;
    }
    for (q = 0; q < p - 1; q++) {
        rA[q] = hb_ref_sm(s->seedA, s->arith_words * i + (uint64_t)q) & s->ring;
        rsum += rA[q];
    }
    rA[p - 1] = (rbit - rsum) & s->ring;
    for (q = 0; q < p; q++) {
        const uint64_t beta = (rA[q] + (q == 0 ? z : 0) - 2 * z * rA[q]) & s->ring;   /* sign = z + r - 2 z r */
        t->drelu[q] = ((q == 0 ? 1 : 0) - beta) & s->ring;
        t->relu[q] = 0;
    }
    if (!want_relu) return;

    /* Beaver multiply x * DReLU */
    const uint64_t base = s->arith_words * i + (uint64_t)(p - 1);
    uint64_t a[HB_REF_MAX_PARTIES], b[HB_REF_MAX_PARTIES], c[HB_REF_MAX_PARTIES];
    uint64_t as = 0, bs = 0, cs = 0, eps = 0, del = 0;
    for (q = 0; q < p; q++) {
        a[q] = hb_ref_sm(s->seedA, base + (uint64_t)q) & s->ring;
        b[q] = hb_ref_sm(s->seedA, base + (uint64_t)(p + q)) & s->ring;
        as += a[q];
        bs += b[q];
    }
    for (q = 0; q < p - 1; q++) {
        c[q] = hb_ref_sm(s->seedA, base + (uint64_t)(2 * p + q)) & s->ring;
        cs += c[q];
    }
    c[p - 1] = (as * bs - cs) & s->ring;
    for (q = 0; q < p; q++) {
        eps += x[q] - a[q];                                  /* opened */
        del += t->drelu[q] - b[q];                           /* opened */
    }
    eps &= s->ring;
    del &= s->ring;
    for (q = 0; q < p; q++) t->relu[q] = (c[q] + eps * b[q] + del * a[q] + (q == 0 ? eps * del : 0)) & s->ring;
}

/* Elements first .. first+n-1.  shares[q] / outs[q] point at party q's element `first`.
 * what: 0 = DReLU shares, 1 = ReLU shares, 2 = XOR shares of the w-bit sum, 3 = XOR shares of the sign,
 * 4 = the sliced shares. */
int hb_ref_mp_eval_range(const int64_t *const *shares, int parties, uint64_t first, uint64_t n, int k, int m,
                         uint64_t seed, int ring_bits, int what, int64_t *const *outs)
{
    mp_shape_t s;
    uint64_t i;
    int q;
    if (what < 0 || what > 4) return HB_REF_EINVAL;
    if (mp_make_shape(&s, parties, k, m, seed, ring_bits) != HB_REF_OK) return HB_REF_EINVAL;
    if (n > 0) {
        if (!shares || !outs) return HB_REF_EINVAL;
        for (q = 0; q < parties; q++)
            if (!shares[q] || !outs[q]) return HB_REF_EINVAL;
    }
    for (i = 0; i < n; i++) {
        uint64_t x[HB_REF_MAX_PARTIES];
        mp_elem_t t;
        for (q = 0; q < parties; q++) x[q] = (uint64_t)shares[q][i];
        mp_eval_element(&s, first + i, x, what == 1, &t);
        const uint64_t *src = what == 0 ? t.drelu : what == 1 ? t.relu : what == 2 ? t.sum : what == 3 ? t.sign : t.u;
        for (q = 0; q < parties; q++) outs[q][i] = (int64_t)src[q];
    }
    return HB_REF_OK;
}

/* Scattered elements: element index[i] of the tensor carries the share values shares[q][i]. */
int hb_ref_mp_eval_at(const int64_t *const *shares, int parties, const uint64_t *index, uint64_t count, int k, int m,
                      uint64_t seed, int ring_bits, int what, int64_t *const *outs)
{
    mp_shape_t s;
    uint64_t i;
    int q;
    if (what < 0 || what > 4) return HB_REF_EINVAL;
    if (mp_make_shape(&s, parties, k, m, seed, ring_bits) != HB_REF_OK) return HB_REF_EINVAL;
    if (count > 0) {
        if (!shares || !outs || !index) return HB_REF_EINVAL;
        for (q = 0; q < parties; q++)
            if (!shares[q] || !outs[q]) return HB_REF_EINVAL;
    }
    for (i = 0; i < count; i++) {
        uint64_t x[HB_REF_MAX_PARTIES];
        mp_elem_t t;
        for (q = 0; q < parties; q++) x[q] = (uint64_t)shares[q][i];
        mp_eval_element(&s, index[i], x, what == 1, &t);
        const uint64_t *src = what == 0 ? t.drelu : what == 1 ? t.relu : what == 2 ? t.sum : what == 3 ? t.sign : t.u;
        for (q = 0; q < parties; q++) outs[q][i] = (int64_t)src[q];
    }
    return HB_REF_OK;
}
