/*
 * hb.h -- C ABI of the reduced-ring secret-shared DReLU / ReLU library for MI355X (gfx950).
 *
 * The operation (paper: "Approximating ReLU on a Reduced Ring for Efficient MPC-based Private
 * Inference"): a tensor x is held as two additive shares on Z_2^64, x = share0 + share1 (mod 2^64),
 * in 2^16 fixed point.  ReLU(x) = x * DReLU(x) (Eq. 1, Eq. 2), and DReLU is evaluated on the slice
 * of bits [k, m) of each share only (Eq. 3; correctness: Sec. 3.1, Theorems 1 and 2):
 *   slice -> arithmetic-to-binary conversion of the two w-bit slices by an adder circuit on XOR
 *   shares whose AND gates consume Beaver triples (Sec. 2.2 "Evaluating ReLU with GMW") -> the most
 *   significant bit is the sign -> binary-to-arithmetic conversion of that one bit, 1 - sign ->
 *   Beaver multiplication with the full 64-bit share.
 * Both parties are evaluated inside one kernel (like the paper's single-node simulator, Sec. 4.1.1);
 * openings are register XOR / add.  All dealer material (AND triples, the B2A bit, the multiply
 * triple) is drawn inside the kernel from two SplitMix64 streams keyed by `seed`.
 *
 * Conventions for every entry point
 *   - (k, m): lowest kept bit, one past the highest kept bit; valid iff 0 <= k < m <= 64; w = m - k.
 *     (The paper writes this slice x[m:k]: its letters are the other way round.)
 *   - share0, share1, out0, out1, out: DEVICE pointers to n contiguous int64, owned by the caller,
 *     8-byte aligned (16-byte alignment is about 2 % faster).  An output may be the very same
 *     buffer as an input (in place); any other overlap between an output and another buffer of the
 *     call is rejected.
 *   - stream: a hipStream_t passed as void* (NULL = the default stream).  Work is enqueued on that
 *     stream; the call does not synchronise, does not allocate and keeps no state between calls.
 *   - opened_bits: HOST pointer or NULL; receives the number of bits the two parties would open to
 *     each other for this call (closed form, written before the call returns).
 *   - return value: HB_OK or a negative status; on error nothing is enqueued and no output is
 *     written.  n == 0 is a successful no-op (arguments are still validated).
 *   - results depend only on (inputs, k, m, seed): the same call twice gives the same shares, and
 *     a tensor may be processed in pieces only through the whole-tensor entry points (element i's
 *     dealer material is indexed by i).
 */
#ifndef HB_H
#define HB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HB_API __attribute__((visibility("default")))

enum hb_status {
    HB_OK = 0,
    HB_EINVAL = -1, /* null pointer with n > 0, bad (k, m), n too large, forbidden overlap, not device memory */
    HB_EALIGN = -2, /* a pointer is not 8-byte aligned */
    HB_EHIP = -3,   /* the HIP runtime refused the launch; hb_last_hip_error() names the reason */
    HB_ENOTSUP = -4, /* this entry point has no kernel for the requested slice width (no entry point returns it today) */
    HB_ETOOBIG = -5  /* hb_relu_party_static: the call needs more workspace than the library's static array holds */
};

/* Largest n accepted by one call (2^40 elements). */
#define HB_MAX_ELEMENTS ((size_t)1 << 40)

/*
 * DReLU (Sec. 2.2; reduced ring: Eq. 3 without the final product).
 * out0[i] + out1[i] = 1 - MSB_w((u0 + u1) mod 2^w) (mod 2^64), u_p = (share_p[i] >> k) mod 2^w:
 * arithmetic shares on Z_2^64 of 1 when the w-bit window of x reads as non-negative, else 0.
 */
HB_API int hb_drelu(const int64_t *share0, const int64_t *share1, size_t n, int k, int m, uint64_t seed,
             int64_t *out0, int64_t *out1, uint64_t *opened_bits, void *stream);

/*
 * Approximate ReLU (Eq. 3): out0[i] + out1[i] = (share0[i] + share1[i]) * DReLU (mod 2^64), where
 * DReLU is exactly what hb_drelu returns for the same (inputs, k, m, seed).
 */
HB_API int hb_relu(const int64_t *share0, const int64_t *share1, size_t n, int k, int m, uint64_t seed,
            int64_t *out0, int64_t *out1, uint64_t *opened_bits, void *stream);

/*
 * The binary half alone (Sec. 2.2: A2B by the adder circuit, sign = most significant bit):
 * out0[i] ^ out1[i] = MSB_w((u0 + u1) mod 2^w); each out_p[i] is 0 or 1 and is party p's XOR share
 * of the sign as it stands after the last prefix round, before B2A.  Same dealer material as
 * hb_drelu / hb_relu.  opened_bits receives n * 2w(1 + 2R) (the circuit's openings only).
 */
HB_API int hb_sign_shares(const int64_t *share0, const int64_t *share1, size_t n, int k, int m, uint64_t seed,
                   int64_t *out0, int64_t *out1, uint64_t *opened_bits, void *stream);

/*
 * Reconstruction (Sec. 2.2 "Notations"): out[i] = share0[i] + share1[i] (mod 2^64) when binary == 0,
 * share0[i] ^ share1[i] otherwise.  `out` may be one of the inputs.
 */
HB_API int hb_open(const int64_t *share0, const int64_t *share1, size_t n, int binary, int64_t *out, void *stream);

/*
 * One tensor of a batched call: the arguments of hb_relu / hb_drelu for that tensor.
 */
typedef struct hb_tensor {
    const int64_t *share0, *share1; /* device, n elements each */
    int64_t *out0, *out1;           /* device, n elements each */
    size_t n;
    int k, m;
    uint64_t seed;                  /* e.g. hb_tensor_seed(root, tensor index) */
} hb_tensor;

/*
 * A set of ReLU layers' tensors in as few launches as possible (the per-layer (k, m) of Sec. 4.2 are
 * fixed offline, so a whole set can be issued at once; one launch per distinct slice width up to 32,
 * up to 24 tensors per launch; wider slices take one launch per tensor).  `tensors` is a HOST array of `count` descriptors, read before the
 * call returns.  The result for every tensor is bit-for-bit what hb_relu (hb_drelu) gives for that
 * tensor alone.  All descriptors are validated before anything is enqueued; besides the per-tensor
 * rules, no output of one tensor may overlap any buffer of another.  opened_bits receives the sum
 * over the tensors.
 */
HB_API int hb_relu_batch(const hb_tensor *tensors, size_t count, uint64_t *opened_bits, void *stream);
HB_API int hb_drelu_batch(const hb_tensor *tensors, size_t count, uint64_t *opened_bits, void *stream);

/*
 * Dealer layouts.  In a prefix round of the adder (Sec. 2.2, Sec. 4.2) both AND gates have the old propagate
 * word P as their first operand.  HB_DEALER_PER_GATE gives every gate its own Beaver triple (the plain reading:
 * 4w opened bits per round).  HB_DEALER_SHARED_MASK lets the two gates of a round share the mask a of P, with
 * triples (a, b, a&b) and (a, b', a&b'): P ^ a is opened once and the round opens 3w bits.  The circuit and
 * every reconstructed value are the same; the individual output shares differ between the layouts.
 * Shared-mask words of one group, in stream order: gate 0 (a_0 a_1 b_0 b_1 c_0); per round a_0 a_1, then
 * b_0 b_1 c_0 of the G-update, then b_0 b_1 c_0 of the P-update; then the B2A word.
 *
 * The *_ex entry points are hb_drelu / hb_relu / hb_relu_batch / hb_drelu_batch with the layout as an argument
 * (`dealer`; any other value is HB_EINVAL); with HB_DEALER_PER_GATE they are those calls bit for bit.
 */
#define HB_DEALER_PER_GATE 0
#define HB_DEALER_SHARED_MASK 1

HB_API int hb_drelu_ex(const int64_t *share0, const int64_t *share1, size_t n, int k, int m, uint64_t seed, int dealer,
                       int64_t *out0, int64_t *out1, uint64_t *opened_bits, void *stream);
HB_API int hb_relu_ex(const int64_t *share0, const int64_t *share1, size_t n, int k, int m, uint64_t seed, int dealer,
                      int64_t *out0, int64_t *out1, uint64_t *opened_bits, void *stream);
HB_API int hb_relu_batch_ex(const hb_tensor *tensors, size_t count, int dealer, uint64_t *opened_bits, void *stream);
HB_API int hb_drelu_batch_ex(const hb_tensor *tensors, size_t count, int dealer, uint64_t *opened_bits, void *stream);

/*
 * A set of tensors prepared once and issued many times (the (k, m) of every ReLU layer are fixed offline, Sec. 4.2,
 * and an inference engine runs the same layers on the same buffers step after step).  hb_plan_create checks the
 * descriptors exactly as hb_relu_batch_ex / hb_drelu_batch_ex do (relu != 0: ReLU, else DReLU; `dealer`: the
 * layout) and records the launches; hb_plan_run only enqueues them on `stream` -- the same kernels, the same
 * result shares -- at a fraction of the host cost per call.  The plan holds device addresses, not memory: the
 * caller keeps the buffers alive and at the same place while the plan is used (contents may change between runs),
 * and the device that was current at creation must be current at every run.  `tensors` is a HOST array read
 * before hb_plan_create returns; *plan receives the handle (host memory owned by the library, released by
 * hb_plan_destroy; NULL on error).  opened_bits (HOST, may be NULL) receives the set's total at every run.
 * A plan may be run from several host threads and on any stream; it is never modified after creation.
 */
typedef struct hb_plan hb_plan;
HB_API int hb_plan_create(const hb_tensor *tensors, size_t count, int relu, int dealer, hb_plan **plan);
HB_API int hb_plan_run(const hb_plan *plan, uint64_t *opened_bits, void *stream);
HB_API void hb_plan_destroy(hb_plan *plan);

/*
 * More than two parties (Sec. 2.2 "Operation of CrypTen": a secret is split into p >= 2 arithmetic shares;
 * Sec. 3.1.2: the two-party analysis carries over).  x[i] = sum over q of shares[q][i] (mod 2^64); every party
 * slices its own share; the p slices are added on XOR shares by a tree of two-operand adder circuits (neighbours
 * (0,1), (2,3), ... level by level); sign, B2A, 1 - sign and the Beaver multiply as for two parties, every triple
 * shared p ways, party 0 adding the public terms:
 *   hb_drelu_mp: sum over q of outs[q][i] = 1 - MSB_w((u_0 + ... + u_{p-1}) mod 2^w),  u_q = (shares[q][i] >> k) mod 2^w
 *   hb_relu_mp : sum over q of outs[q][i] = x[i] * that value.
 * Dealer layout: an AND gate owns 3p-1 words a_0..a_{p-1} b_0..b_{p-1} c_0..c_{p-2}; gate t of adder s (adders in
 * evaluation order) starts at word (s(1+2R) + t)(3p-1) of its group; a group owns (p-1)(1+2R)(3p-1) + 1 words, the
 * last one holding the B2A bits (bit p*j + q: party q, lane j), so a group has L = min(floor(64/w), floor(64/p))
 * elements; element i owns the 4p-2 arithmetic words rA_0..rA_{p-2} | a_0..a_{p-1} | b_0..b_{p-1} | c_0..c_{p-2}.
 * With parties == 2 the calls are hb_drelu / hb_relu bit for bit.
 *
 * shares, outs: HOST arrays of `parties` DEVICE pointers (n int64 each, same rules as hb_relu: 8-byte aligned, an
 * output may be exactly one of the inputs, no other overlap).  parties: 2, 3 or 4 (HB_EINVAL otherwise).
 * opened_bits receives what ONE party sends to ONE other party: n * ((p-1) * 2w(1+2R) + 1) (+ 128 n for ReLU).
 */
#define HB_MAX_PARTIES 4
HB_API int hb_drelu_mp(const int64_t *const *shares, int parties, size_t n, int k, int m, uint64_t seed,
                       int64_t *const *outs, uint64_t *opened_bits, void *stream);
HB_API int hb_relu_mp(const int64_t *const *shares, int parties, size_t n, int k, int m, uint64_t seed,
                      int64_t *const *outs, uint64_t *opened_bits, void *stream);
HB_API uint64_t hb_opened_bits_mp(int relu, int parties, int k, int m, size_t n);   /* 0 for invalid arguments */

/*
 * Party-faithful ReLU: the same protocol and dealer material as hb_relu, but every opening goes through
 * memory the way it would go over the link between two GPUs (Sec. 2.2: each AND, the B2A and the multiply
 * open masked values; Sec. 4.2: the w-bit fields are packed into 64-bit words before each communication).
 * Each party is evaluated by its own threads, owns its state and writes the words it sends to its "wire";
 * a party reads the other wire only for completed rounds (one kernel launch per communication round:
 * slice + gate 0, R prefix rounds, sign, B2A bits, multiply openings, result).  out0 / out1 are
 * bit-for-bit the shares hb_relu returns.
 *
 * Wire of party p, 64-bit words: [2G: gate 0][4G per round, R rounds][ceil(n/64): B2A][2n: multiply], G =
 * ceil(n / L) groups of L = min(floor(64/w), 32) elements; in a group word field j sits at bit j*w; word
 * [2g] / [4g + 0, 2] holds the masked first operand, [2g + 1] / [4g + 1, 3] the masked second operand of the
 * gate(s); B2A bit i%64 of word i/64 belongs to element i; multiply words [2i], [2i+1] are x_p - a_p and
 * DReLU_p - b_p.  Bits that belong to no element are zero.  hb_party_wire_words gives the word count
 * (8 bytes each; 64 x words = opened bits when w*L = 64 and 64 divides n).
 *
 * workspace: DEVICE memory, 256-byte aligned, hb_party_workspace_bytes(n, k, m) bytes, not overlapping any
 * other buffer of the call; after the call the wires are at byte offsets hb_party_wire_offset(n, k, m, p).
 * Inputs and outputs must not overlap each other here (in place is not supported).  wire_bytes (HOST, may
 * be NULL) receives the bytes each party wrote to its wire.
 */
HB_API int hb_relu_party(const int64_t *share0, const int64_t *share1, size_t n, int k, int m, uint64_t seed,
                         int64_t *out0, int64_t *out1, void *workspace, size_t workspace_bytes,
                         uint64_t *wire_bytes, void *stream);
HB_API size_t hb_party_workspace_bytes(size_t n, int k, int m);  /* 0 for an invalid (k, m) or n too large */

/*
 * hb_relu_party for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same result shares and the same
 * wire traffic as hb_relu_party, but the workspace is an array of HB_PARTY_STATIC_BYTES bytes that lives inside
 * the library's code object on every GPU the library runs on (held until the process ends).  The call allocates
 * nothing and frees nothing; its first call on a device looks the array's device address up (once per device) --
 * make that first call outside any stream capture.
 *   - accepted sizes: hb_party_workspace_bytes(n, k, m) <= HB_PARTY_STATIC_BYTES (about 796,000 elements at
 *     w = 8, 127,000 at w = 64); larger calls return HB_ETOOBIG and enqueue nothing.
 *   - all calls on one GPU share that GPU's array: it keeps the previous call's contents (every word a call reads
 *     it has written itself, so nothing needs clearing), and two calls whose kernels may overlap in time -- on
 *     different streams, or from different threads -- race.  Order them on one stream or with events.
 *   - the wires stay inside the library; wire_bytes (HOST, may be NULL) receives the bytes each party wrote.
 * Everything else (arguments, errors, no in-place operation) is as for hb_relu_party.
 */
#define HB_PARTY_STATIC_BYTES ((size_t)64 << 20)
HB_API int hb_relu_party_static(const int64_t *share0, const int64_t *share1, size_t n, int k, int m, uint64_t seed,
                                int64_t *out0, int64_t *out1, uint64_t *wire_bytes, void *stream);
HB_API size_t hb_party_wire_words(size_t n, int k, int m);
HB_API size_t hb_party_wire_offset(size_t n, int k, int m, int party);

/*
 * The same on a dealer layout (`dealer` as for hb_relu_ex; HB_DEALER_PER_GATE is hb_relu_party bit for bit).  On
 * HB_DEALER_SHARED_MASK the two gates of a prefix round share the mask of P, so each party sends P ^ a once: a round
 * occupies three wire words per group, [3g] the masked P, [3g + 1] the masked second operand of the G-update,
 * [3g + 2] that of the P-update, and the wire is [2G][3G per round, R rounds][ceil(n/64)][2n] words -- 64 x words =
 * hb_opened_bits_ex(1, k, m, n, HB_DEALER_SHARED_MASK) when w*L = 64 and 64 divides n.  Result shares equal
 * hb_relu_ex's for that layout.  The *_ex size queries return 0 for an unknown layout.
 */
HB_API int hb_relu_party_ex(const int64_t *share0, const int64_t *share1, size_t n, int k, int m, uint64_t seed,
                            int dealer, int64_t *out0, int64_t *out1, void *workspace, size_t workspace_bytes,
                            uint64_t *wire_bytes, void *stream);
HB_API size_t hb_party_workspace_bytes_ex(size_t n, int k, int m, int dealer);
HB_API size_t hb_party_wire_words_ex(size_t n, int k, int m, int dealer);
HB_API size_t hb_party_wire_offset_ex(size_t n, int k, int m, int dealer, int party);

/*
 * Float boundary of the single-node simulator (Sec. 4.1.1: floating-point activations are converted to ring
 * elements, shared, and the ReLU layer is evaluated by the protocol).  Fixed point is x = round(2^16 x_f), ties
 * to even (Sec. 2.2, Sec. 3.1); NaN encodes as 0 and |2^16 x_f| is clamped to 2^62.
 *   hb_share_f32 : share0[i] = output i of the SplitMix64 stream started at share_seed (uniform on Z_2^64),
 *                  share1[i] = round(2^16 x[i]) - share0[i].
 *   hb_reveal_f32: y[i] = (float)((share0[i] + share1[i] mod 2^64, read as signed) / 2^16).
 *   hb_sim_relu_f32: y = hb_reveal_f32(hb_relu(hb_share_f32(x, share_seed), k, m, seed)) in ONE kernel that
 *                  reads 4 bytes and writes 4 bytes per element; bit-identical to the composition, for every
 *                  slice width; y may be x itself.
 * x, y: device float arrays (4-byte aligned; 8-byte aligned for hb_sim_relu_f32).
 */
HB_API int hb_share_f32(const float *x, size_t n, uint64_t share_seed, int64_t *share0, int64_t *share1, void *stream);
HB_API int hb_reveal_f32(const int64_t *share0, const int64_t *share1, size_t n, float *y, void *stream);
HB_API int hb_sim_relu_f32(const float *x, size_t n, int k, int m, uint64_t seed, uint64_t share_seed, float *y,
                           void *stream);

/*
 * Zero-error search for the high cut (Sec. 4.1.2, the "eco" strategy: try every high cut with no low cut
 * and see whether any DReLU result changes).  counts[m - 1] receives the number of elements whose DReLU
 * on the slice [0, m) differs from DReLU on the full ring, for m = 1 .. 64 (counts[63] is always 0).
 * share0, share1: device, n int64 each.  counts: DEVICE pointer to 64 uint64 (8-byte aligned), overwritten;
 * it must not overlap the shares.  Two kernels are enqueued on `stream` (clear, then scan).
 */
HB_API int hb_eco_scan(const int64_t *share0, const int64_t *share1, size_t n, uint64_t *counts, void *stream);

/*
 * The eco choice from a scan: the smallest m such that no m' >= m has a mismatch, i.e. the fewest bits
 * [0, m) that reproduce the full-ring DReLU on every scanned element (Theorem 1).  counts: HOST pointer
 * to the 64 values read back from hb_eco_scan.  Returns m in [1, 64], or HB_EINVAL for a null pointer.
 */
HB_API int hb_eco_choose(const uint64_t *counts);

/* Seed of tensor `tensor_id` in a set of tensors keyed by one root seed (host-only, no GPU work). */
HB_API uint64_t hb_tensor_seed(uint64_t root_seed, uint64_t tensor_id);

/*
 * Bits opened for n elements: n * (2w(1 + 2R) + 1) for DReLU (relu == 0), plus 128 n for ReLU
 * (relu != 0); R = 0 if w == 1 else ceil(log2 w) rounds (Sec. 4.2).  The unpacked 64-bit baseline
 * of Sec. 2.3 is 29 * 64 = 1856 bits per element.  Returns 0 for an invalid (k, m).
 */
HB_API uint64_t hb_opened_bits(int relu, int k, int m, size_t n);

/* The same count for a dealer layout: HB_DEALER_SHARED_MASK opens n * (2w + 3wR + 1) (+ 128 n).  0 for an unknown layout. */
HB_API uint64_t hb_opened_bits_ex(int relu, int k, int m, size_t n, int dealer);

/* Static description of a status code. */
HB_API const char *hb_strerror(int status);

/* Text of the HIP error behind the calling thread's most recent HB_EHIP ("" if none). */
HB_API const char *hb_last_hip_error(void);

#ifdef __cplusplus
}
#endif

#endif /* HB_H */
