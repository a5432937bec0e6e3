// Kernels of the fused path: both parties of an element live in one thread and every opening stays in registers.
//
//   group_kernel       one thread per group of L = min(64/W, 32) consecutive elements: packs the slices of its
//                      elements into two SWAR words, runs the circuit (gate 0, all prefix rounds, sign), then
//                      finishes its elements one by one (B2A, Beaver multiply).  No LDS.  Used for w > 32.
//   tile_kernel        one wavefront per 64 groups (32 for w <= 3), coalesced 16-byte memory traffic per lane, slices and sign
//   tile_batch_kernel  words exchanged through wave-private LDS (described above the kernel).  The batch form
//                      serves several tensors of one width; tile_sim_kernel is the float-in / float-out form.
//   open_kernel        share0 + share1 or share0 ^ share1.
//
// Nothing but the input shares is read from memory and nothing but the output shares is written: the algorithmic
// traffic is 32 bytes per element (24 for open_kernel, 8 for tile_sim_kernel).
#pragma once

#include <type_traits>

#include "hb_protocol.hpp"

namespace hb {

constexpr int kBlock = 256;

struct alignas(16) U64x2 {
    uint64_t a, b;
};

// Memory accesses with the non-temporal hint: every share is read once and every result written once, so
// nothing is worth keeping in the caches (streaming 2-in / 2-out traffic runs about a tenth faster with it).
// A pair of elements travels as one 16-byte access; the type only promises the 8-byte alignment the interface
// requires (the hardware takes 16-byte global accesses at any 4-byte alignment).
typedef uint64_t u64x2_t __attribute__((ext_vector_type(2), aligned(8)));
__device__ __forceinline__ U64x2 load_stream2(const uint64_t *p)
{
    const u64x2_t v = __builtin_nontemporal_load(reinterpret_cast<const u64x2_t *>(p));
    return U64x2{v.x, v.y};
}
__device__ __forceinline__ void store_stream2(uint64_t *p, U64x2 v)
{
    __builtin_nontemporal_store(u64x2_t{v.a, v.b}, reinterpret_cast<u64x2_t *>(p));
}
__device__ __forceinline__ uint64_t load_stream(const uint64_t *p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ void store_stream(uint64_t *p, uint64_t v) { __builtin_nontemporal_store(v, p); }

template <int W, int MODE, bool VEC>
__global__ void __launch_bounds__(kBlock)
group_kernel(const uint64_t *x0, const uint64_t *x1, uint64_t n, uint64_t groups, int k, uint64_t seedB,
             uint64_t seedA, uint64_t *o0, uint64_t *o1)
{
    using S = Shape<W>;
    constexpr int L = S::L;
    // keep the loaded shares in registers across the circuit when that is cheap, else read them again
    constexpr bool kHold = (op_of(MODE) == kRelu) && (L <= 8);

    const uint64_t g = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (g >= groups) return;
    const uint64_t i0 = g * (uint64_t)L;
    const bool full = (n - i0) >= (uint64_t)L;
    const int cnt = full ? L : (int)(n - i0);

    uint64_t xa[kHold ? L : 1], xb[kHold ? L : 1];
    uint64_t u0 = 0, u1 = 0;

    if (VEC && full && (L % 2 == 0)) {
#pragma unroll
        for (int j = 0; j < L / 2; ++j) {
            const U64x2 a = load_stream2(x0 + i0 + 2 * j), b = load_stream2(x1 + i0 + 2 * j);
            u0 |= ((a.a >> k) & S::kField) << ((2 * j) * W % 64);
            u0 |= ((a.b >> k) & S::kField) << ((2 * j + 1) * W % 64);
            u1 |= ((b.a >> k) & S::kField) << ((2 * j) * W % 64);
            u1 |= ((b.b >> k) & S::kField) << ((2 * j + 1) * W % 64);
            if (kHold) {
                xa[2 * j] = a.a;
                xa[2 * j + 1] = a.b;
                xb[2 * j] = b.a;
                xb[2 * j + 1] = b.b;
            }
        }
    } else {
#pragma unroll
        for (int j = 0; j < L; ++j) {
            uint64_t a = 0, b = 0;
            if (j < cnt) {
                a = load_stream(x0 + i0 + j);
                b = load_stream(x1 + i0 + j);
            }
            u0 |= ((a >> k) & S::kField) << (j * W % 64);
            u1 |= ((b >> k) & S::kField) << (j * W % 64);
            if (kHold) {
                xa[j] = a;
                xb[j] = b;
            }
        }
    }

    const uint64_t zg = seedB + (g * (uint64_t)S::words_per_group(shared_of(MODE)) + 1) * kGamma;
    const Pair sum = a2b_sum<W, shared_of(MODE)>(u0, u1, zg);
    uint64_t wb = 0;
    if (op_of(MODE) != kSign) wb = mix64(zg + (uint64_t)S::b2a_word(shared_of(MODE)) * kGamma);

    const uint64_t zA0 = seedA + (6 * i0 + 1) * kGamma;
    if (VEC && full && (L % 2 == 0)) {
#pragma unroll
        for (int j = 0; j < L / 2; ++j) {
            Pair xe{0, 0}, xo{0, 0};
            if (op_of(MODE) == kRelu) {
                if (kHold) {
                    xe = Pair{xa[2 * j], xb[2 * j]};
                    xo = Pair{xa[2 * j + 1], xb[2 * j + 1]};
                } else {
                    const U64x2 a = load_stream2(x0 + i0 + 2 * j);
                    const U64x2 b = load_stream2(x1 + i0 + 2 * j);
                    xe = Pair{a.a, b.a};
                    xo = Pair{a.b, b.b};
                }
            }
            const Pair re = finish_element<W, MODE>(sum, wb, 2 * j, xe, zA0 + (uint64_t)(6 * (2 * j)) * kGamma);
            const Pair ro = finish_element<W, MODE>(sum, wb, 2 * j + 1, xo, zA0 + (uint64_t)(6 * (2 * j + 1)) * kGamma);
            store_stream2(o0 + i0 + 2 * j, U64x2{re.p0, ro.p0});
            store_stream2(o1 + i0 + 2 * j, U64x2{re.p1, ro.p1});
        }
    } else {
#pragma unroll
        for (int j = 0; j < L; ++j) {
            if (j < cnt) {
                Pair x{0, 0};
                if (op_of(MODE) == kRelu) x = kHold ? Pair{xa[j], xb[j]} : Pair{load_stream(x0 + i0 + j), load_stream(x1 + i0 + j)};
                const Pair r = finish_element<W, MODE>(sum, wb, j, x, zA0 + (uint64_t)(6 * j) * kGamma);
                store_stream(o0 + i0 + j, r.p0);
                store_stream(o1 + i0 + j, r.p1);
            }
        }
    }
}

// out = share0 + share1 (mod 2^64) or share0 ^ share1; two elements per thread when VEC.
template <bool VEC>
__global__ void __launch_bounds__(kBlock)
open_kernel(const uint64_t *x0, const uint64_t *x1, uint64_t n, int binary, uint64_t *out)
{
    const uint64_t t = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (VEC) {
        const uint64_t i = 2 * t;
        if (i + 1 < n) {
            const U64x2 a = load_stream2(x0 + i);
            const U64x2 b = load_stream2(x1 + i);
            store_stream2(out + i, binary ? U64x2{a.a ^ b.a, a.b ^ b.b} : U64x2{a.a + b.a, a.b + b.b});
        } else if (i < n) {
            const uint64_t a = load_stream(x0 + i), b = load_stream(x1 + i);
            store_stream(out + i, binary ? (a ^ b) : (a + b));
        }
    } else {
        if (t < n) {
            const uint64_t a = load_stream(x0 + t), b = load_stream(x1 + t);
            store_stream(out + t, binary ? (a ^ b) : (a + b));
        }
    }
}


// ------------------------------------------------------------------------------------------------
// Tile kernel (slice widths up to 32).
//
// A wavefront owns a tile of 64*L consecutive elements = 64 groups (32 groups when L > 16).  Memory traffic and the
// per-element arithmetic are laid out for coalescing: lane l loads / finishes / stores the element
// pairs (2(c*64 + l), +1), so every load and store instruction of the wave covers 1 KiB of
// consecutive addresses.  The circuit is laid out for dealer-word sharing: lane l evaluates group l
// of the tile.  The two layouts meet in the wave's private piece of LDS: owners deposit the sliced
// shares of their elements, group lanes collect the L fields of their group, and after the circuit
// each group lane leaves its sign shares and B2A dealer word for the owners of its elements.
// All exchange stays inside one wavefront, whose LDS operations execute in program order, so no
// workgroup barrier is needed; wave_sync() only keeps the compiler from moving LDS accesses across.
// ------------------------------------------------------------------------------------------------

constexpr int kWave = 64;
constexpr int kWavesPerBlock = kBlock / kWave;

__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Geometry of a wave-tile for slice width w, shared by the kernels and the host code that counts tiles.
// A wavefront takes 64 groups, or 32 when a group has more than 16 elements (w <= 3): a lane then still owns
// at most 8 element pairs, which is what fits in registers, and only the lower half of the lanes runs the
// (short) circuit.
constexpr int tile_lanes_per_word(int w) { return 64 / w > 32 ? 32 : 64 / w; }
constexpr int tile_groups(int w) { return tile_lanes_per_word(w) > 16 ? 32 : 64; }
constexpr int tile_elements(int w) { return tile_groups(w) * tile_lanes_per_word(w); }

template <int W>
struct TileTraits {
    using S = Shape<W>;
    static constexpr int L = S::L;
    static constexpr bool kSupported = (L >= 2);                // every width below 33
    // the group lane publishes party 1's sign bit of a field next to party 0's; one-bit fields have no room for
    // that, but their 32 fields leave the upper half of the word free
    static constexpr int kSign1 = (W == 1) ? 32 : 1;
    static constexpr int kGroups = tile_groups(W);              // groups per wavefront
    static constexpr int kTile = tile_elements(W);              // elements per wavefront
    static constexpr int kPairs = (kTile / 2 + kWave - 1) / kWave;   // element pairs per lane (the last may be idle)
    // W in {4, 8, 16, 32}: a pair of fields is an addressable LDS item (1, 2, 4, 8 bytes), so owners can
    // write their pair straight into the group's packed word.  Other widths go through one entry per element.
    static constexpr bool kPacked = (W == 4 || W == 8 || W == 16 || W == 32);
    using Item = typename std::conditional<(W == 4), uint8_t,
                 typename std::conditional<(W == 8), uint16_t,
                 typename std::conditional<(W == 16), uint32_t, uint64_t>::type>::type>::type;
    static constexpr int kHalf = (W <= 16) ? 16 : 32;           // bits per party inside an unpacked LDS entry
    using Entry = typename std::conditional<(W <= 16), uint32_t, uint64_t>::type;
    // LDS bytes per wavefront for the slices
    static constexpr int kSliceBytes = kPacked ? 2 * kWave * 8 : kTile * (int)sizeof(Entry);
};

// ---- where a tile's element pairs come from and where the results go ----------------------------------------
// Shares in, shares out: the library's normal boundary.
// Element i = tile0 + e: tile0 (the tile's first element) is uniform over the wavefront, e is the lane's
// 32-bit offset inside the tile, so an address is a scalar base plus a 32-bit vector offset.
struct ShareIO {
    const uint64_t *x0, *x1;
    uint64_t *o0, *o1;
    template <bool FULL>
    __device__ __forceinline__ void load_pair(uint64_t tile0, unsigned e, uint64_t n, U64x2 &a, U64x2 &b) const
    {
        const uint64_t *t0 = x0 + tile0, *t1 = x1 + tile0;
        if (FULL || tile0 + e + 1 < n) {
            a = load_stream2(t0 + e);
            b = load_stream2(t1 + e);
        } else if (tile0 + e < n) {
            a.a = load_stream(t0 + e);
            b.a = load_stream(t1 + e);
        }
    }
    template <bool FULL>
    __device__ __forceinline__ void store_pair(uint64_t tile0, unsigned e, uint64_t n, Pair r0, Pair r1) const
    {
        uint64_t *t0 = o0 + tile0, *t1 = o1 + tile0;
        if (FULL || tile0 + e + 1 < n) {
            store_stream2(t0 + e, U64x2{r0.p0, r1.p0});
            store_stream2(t1 + e, U64x2{r0.p1, r1.p1});
        } else if (tile0 + e < n) {
            store_stream(t0 + e, r0.p0);
            store_stream(t1 + e, r0.p1);
        }
    }
};

// Fixed point of the paper's setting (Sec. 2.2 "Operation of CrypTen", Sec. 3.1): x = round(2^16 x_f),
// ties to even; NaN encodes as 0 and magnitudes are clamped to 2^62 so the conversion is defined for every float.
__host__ __device__ __forceinline__ uint64_t encode_fixed16(float v)
{
    double d = (double)v * 65536.0;
    if (!(d == d)) d = 0.0;
    d = d > 0x1p62 ? 0x1p62 : (d < -0x1p62 ? -0x1p62 : d);
#if defined(__HIP_DEVICE_COMPILE__)
    return (uint64_t)__double2ll_rn(d);
#else
    return (uint64_t)(long long)__builtin_rint(d);
#endif
}

__host__ __device__ __forceinline__ float decode_fixed16(uint64_t v)
{
    return (float)((double)(int64_t)v * (1.0 / 65536.0));
}

struct alignas(8) F32x2 {
    float a, b;
};

// Plaintext floats in, plaintext floats out (the single-node simulator of Sec. 4.1.1): the load encodes to fixed
// point and shares additively with share0[i] = output i of the SplitMix64 stream started at seedS; the store opens
// the two result shares and decodes.  Nothing but 4 bytes per element travels each way.
struct FloatIO {
    const float *x;
    float *y;
    uint64_t seedS;
    template <bool FULL>
    __device__ __forceinline__ void load_pair(uint64_t tile0, unsigned e, uint64_t n, U64x2 &a, U64x2 &b) const
    {
        const uint64_t i = tile0 + e;
        const float *t = x + tile0;
        float f0 = 0.0f, f1 = 0.0f;
        if (FULL || i + 1 < n) {
            const F32x2 v = *reinterpret_cast<const F32x2 *>(t + e);
            f0 = v.a;
            f1 = v.b;
        } else if (i < n) {
            f0 = t[e];
        } else {
            return;
        }
        const uint64_t z = seedS + (i + 1) * kGamma;
        a.a = mix64(z);
        a.b = mix64(z + kGamma);
        b.a = encode_fixed16(f0) - a.a;
        b.b = encode_fixed16(f1) - a.b;
    }
    template <bool FULL>
    __device__ __forceinline__ void store_pair(uint64_t tile0, unsigned e, uint64_t n, Pair r0, Pair r1) const
    {
        float *t = y + tile0;
        if (FULL || tile0 + e + 1 < n) {
            *reinterpret_cast<F32x2 *>(t + e) = F32x2{decode_fixed16(r0.p0 + r0.p1), decode_fixed16(r1.p0 + r1.p1)};
        } else if (tile0 + e < n) {
            t[e] = decode_fixed16(r0.p0 + r0.p1);
        }
    }
};

// Work of one wavefront on wave-tile `tile` of one tensor.  slice_lds / verdict: this wave's LDS.  FULL: the
// whole tile lies inside the tensor, so no access needs a bounds check (every tile but a tensor's last).
template <int W, int MODE, bool FULL, class IO>
__device__ __forceinline__ void tile_body_impl(const IO &io, uint64_t n, int k, uint64_t seedB, uint64_t seedA,
                                               uint64_t tile, int lane, unsigned char *slice_lds, U64x2 *verdict)
{
    using T = TileTraits<W>;
    using S = Shape<W>;
    constexpr int L = T::L;
    static_assert(T::kSupported, "tile kernel needs W <= 32");
    const uint64_t tile0 = tile * T::kTile;

    // ---- owners: load, slice, deposit -------------------------------------------------------
    U64x2 xa[T::kPairs], xb[T::kPairs];
#pragma unroll
    for (int c = 0; c < T::kPairs; ++c) {
        const int pr = c * kWave + lane;     // pair index inside the tile
        const int e = 2 * pr;
        xa[c] = U64x2{0, 0};
        xb[c] = U64x2{0, 0};
        if (e < T::kTile) {
            io.template load_pair<FULL>(tile0, (unsigned)e, n, xa[c], xb[c]);
            if constexpr (T::kPacked) {
                // the pair's two fields of party 0 / party 1, already at their place relative to the pair
                using Item = typename T::Item;
                Item *w0 = reinterpret_cast<Item *>(slice_lds);
                Item *w1 = reinterpret_cast<Item *>(slice_lds + kWave * 8);
                w0[pr] = (Item)(((xa[c].a >> k) & S::kField) | (((xa[c].b >> k) & S::kField) << (W % 64)));
                w1[pr] = (Item)(((xb[c].a >> k) & S::kField) | (((xb[c].b >> k) & S::kField) << (W % 64)));
            } else {
                using Entry = typename T::Entry;
                Entry *slices = reinterpret_cast<Entry *>(slice_lds);
                slices[e] = (Entry)((xa[c].a >> k) & S::kField) | ((Entry)((xb[c].a >> k) & S::kField) << T::kHalf);
                slices[e + 1] = (Entry)((xa[c].b >> k) & S::kField) | ((Entry)((xb[c].b >> k) & S::kField) << T::kHalf);
            }
        }
    }
    wave_sync();

    // ---- group lanes: collect fields, run the circuit, publish the verdict ----------------------
    if (T::kGroups == kWave || lane < T::kGroups) {
        uint64_t u0 = 0, u1 = 0;
        if constexpr (T::kPacked) {
            u0 = reinterpret_cast<const uint64_t *>(slice_lds)[lane];
            u1 = reinterpret_cast<const uint64_t *>(slice_lds + kWave * 8)[lane];
        } else {
            using Entry = typename T::Entry;
            const Entry *slices = reinterpret_cast<const Entry *>(slice_lds);
#pragma unroll
            for (int j = 0; j < L; ++j) {
                const Entry en = slices[lane * L + j];
                u0 |= (uint64_t)(en & (Entry)S::kField) << (j * W);
                u1 |= (uint64_t)(en >> T::kHalf) << (j * W);
            }
        }
        const uint64_t g = tile * T::kGroups + lane;
        const uint64_t zg = seedB + (g * (uint64_t)S::words_per_group(shared_of(MODE)) + 1) * kGamma;
        const Pair sum = a2b_sum<W, shared_of(MODE)>(u0, u1, zg);
        // sign of field j: party 0 at bit jW, party 1 at bit jW + kSign1
        const uint64_t ones = S::ones();
        const uint64_t sg = ((sum.p0 >> (W - 1)) & ones) | (((sum.p1 >> (W - 1)) & ones) << T::kSign1);
        uint64_t wb = 0;
        if (op_of(MODE) != kSign) wb = mix64(zg + (uint64_t)S::b2a_word(shared_of(MODE)) * kGamma);
        verdict[lane] = U64x2{sg, wb};
    }
    wave_sync();

    // ---- owners: pick up the verdict of each element's group, finish, store ---------------------
    const uint64_t zA0 = seedA + (6 * (tile0 + 2 * (uint64_t)lane) + 1) * kGamma;   // A[6i] of the lane's first element
#pragma unroll
    for (int c = 0; c < T::kPairs; ++c) {
        const int e = 2 * (c * kWave + lane);
        if (e < T::kTile) {
            Pair r[2];
            const int grp0 = e / L, j0 = e - grp0 * L;
            const U64x2 v0 = verdict[grp0];
            // both elements of the pair sit in one group unless L is odd and the pair straddles two
            const bool split = (L % 2 != 0) && (j0 == L - 1);
            const U64x2 v1 = split ? verdict[grp0 + 1] : v0;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const U64x2 v = h ? v1 : v0;
                const int j = h ? (split ? 0 : j0 + 1) : j0;
                // only two bits of each shifted word are used
                const uint64_t sg = v.a >> (j * W);
                const Pair sign{sg & 1u, (sg >> T::kSign1) & 1u};
                if (op_of(MODE) == kSign) {
                    r[h] = sign;
                } else {
                    const uint32_t rh = (uint32_t)(v.b >> (2 * j));
                    const Pair rho{rh & 1u, (rh >> 1) & 1u};
                    const uint64_t zA = zA0 + (uint64_t)(6 * (2 * c * kWave + h)) * kGamma;
                    const Pair D = b2a_drelu(sign, rho, zA);
                    r[h] = (op_of(MODE) == kDrelu) ? D : beaver_mul(Pair{h ? xa[c].b : xa[c].a, h ? xb[c].b : xb[c].a}, D, zA);
                }
            }
            io.template store_pair<FULL>(tile0, (unsigned)e, n, r[0], r[1]);
        }
    }
}

// `tile` must be uniform over the wavefront (callers derive it from wave_index()).
template <int W, int MODE, class IO>
__device__ __forceinline__ void tile_body(const IO &io, uint64_t n, int k, uint64_t seedB, uint64_t seedA,
                                          uint64_t tile, int lane, unsigned char *slice_lds, U64x2 *verdict)
{
    if ((tile + 1) * TileTraits<W>::kTile <= n)
        tile_body_impl<W, MODE, true>(io, n, k, seedB, seedA, tile, lane, slice_lds, verdict);
    else
        tile_body_impl<W, MODE, false>(io, n, k, seedB, seedA, tile, lane, slice_lds, verdict);
}

// The wavefront's number inside its workgroup, as a scalar: everything derived from it (tile number, tensor
// descriptor, base addresses) then stays in scalar registers.
__device__ __forceinline__ int wave_index()
{
    return __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
}

template <int W, int MODE>
__global__ void __launch_bounds__(kBlock)
tile_kernel(const uint64_t *x0, const uint64_t *x1, uint64_t n, int k, uint64_t seedB, uint64_t seedA, uint64_t *o0,
            uint64_t *o1)
{
    using T = TileTraits<W>;
    __shared__ __attribute__((aligned(16))) unsigned char slices_all[kWavesPerBlock][T::kSliceBytes];
    __shared__ U64x2 verdict_all[kWavesPerBlock][kWave];     // per group: {sign shares, B2A dealer word}
    const int lane = threadIdx.x % kWave, wv = wave_index();
    const uint64_t tile = (uint64_t)blockIdx.x * kWavesPerBlock + wv;
    if (tile * T::kTile >= n) return;        // whole wavefront beyond the tensor (uniform per wave)
    tile_body<W, MODE>(ShareIO{x0, x1, o0, o1}, n, k, seedB, seedA, tile, lane, slices_all[wv], verdict_all[wv]);
}

// Several tensors of one slice width in a single launch.  The descriptors travel in the kernel
// argument block; wave-tiles of all tensors are numbered consecutively and tile_end[t] is the number
// of wave-tiles in tensors 0..t.
constexpr int kBatchMax = 24;

struct BatchTensor {
    const uint64_t *x0, *x1;
    uint64_t *o0, *o1;
    uint64_t n, seedB, seedA;
    int k, pad;
};

struct BatchArgs {
    int count, pad;
    uint64_t tile_end[kBatchMax];
    BatchTensor t[kBatchMax];
};

template <int W, int MODE>
__global__ void __launch_bounds__(kBlock)
tile_batch_kernel(const BatchArgs args)
{
    using T = TileTraits<W>;
    __shared__ __attribute__((aligned(16))) unsigned char slices_all[kWavesPerBlock][T::kSliceBytes];
    __shared__ U64x2 verdict_all[kWavesPerBlock][kWave];
    const int lane = threadIdx.x % kWave, wv = wave_index();
    const uint64_t gt = (uint64_t)blockIdx.x * kWavesPerBlock + wv;          // wave-tile number over the whole batch
    if (gt >= args.tile_end[args.count - 1]) return;
    int ti = 0;
    while (gt >= args.tile_end[ti]) ++ti;                                     // uniform per wave, at most kBatchMax steps
    const uint64_t tile = gt - (ti ? args.tile_end[ti - 1] : 0);
    const BatchTensor &d = args.t[ti];
    tile_body<W, MODE>(ShareIO{d.x0, d.x1, d.o0, d.o1}, d.n, d.k, d.seedB, d.seedA, tile, lane, slices_all[wv], verdict_all[wv]);
}

// ------------------------------------------------------------------------------------------------
// Small wave-tile (short tensors): 16 groups per wavefront and four lanes per group.
//
// When a launch has fewer wave-tiles than the chip has SIMDs, its duration is one wavefront's serial instruction
// stream (about 2000 vector instructions at w = 8), most of it dealer words.  Here a wavefront takes a quarter of
// the elements and the four lanes of a group split the group's dealer words between them (every fourth word
// each), hand them to one another through LDS, and all evaluate the (short) gate logic; owners then finish one
// element pair per lane (at w = 8) instead of four.  Same dealer indices, same results; about a third of the
// serial work per wavefront, about 1.25 times the total work, so this form is used only for launches that
// cannot fill the chip.  Standard dealer layout, DReLU and ReLU, 4 <= w <= 32.
// ------------------------------------------------------------------------------------------------
template <int W>
struct SmallTraits {
    using S = Shape<W>;
    using T = TileTraits<W>;
    static constexpr int L = S::L;
    static constexpr bool kSupported = T::kSupported && (W >= 4);
    static constexpr int kSplit = 4;                            // lanes per group
    static constexpr int kGroups = kWave / kSplit;              // groups per wavefront
    static constexpr int kTile = kGroups * L;                   // elements per wavefront
    static constexpr int kPairs = (kTile / 2 + kWave - 1) / kWave;
    static constexpr int kWords = 10 * S::R + 1;                // evaluated dealer words of a group: 2R gates + B2A
    static constexpr int kWordsPerLane = (kWords + kSplit - 1) / kSplit;
    // words of LDS per group: a multiple of 32 words plus 2, so that the 16 groups' 16-byte reads of one word
    // fall into 16 different sets of four banks (and the stride stays a 16-byte multiple)
    static constexpr int kStride = ((kWords + 31) / 32) * 32 + 2;
    static constexpr int kSliceBytes = T::kPacked ? 2 * kGroups * 8 : kTile * (int)sizeof(typename T::Entry);
};

constexpr int small_tile_elements(int w) { return 16 * tile_lanes_per_word(w); }

template <int W, int MODE, bool FULL>
__device__ __forceinline__ void small_tile_body_impl(const ShareIO &io, uint64_t n, int k, uint64_t seedB, uint64_t seedA,
                                                     uint64_t tile, int lane, unsigned char *slice_lds, uint64_t *words_lds,
                                                     U64x2 *verdict)
{
    using T = TileTraits<W>;
    using Q = SmallTraits<W>;
    using S = Shape<W>;
    constexpr int L = Q::L;
    static_assert(Q::kSupported && !shared_of(MODE) && op_of(MODE) != kSign, "small tiles: standard layout, DReLU / ReLU");
    const uint64_t tile0 = tile * Q::kTile;

    // ---- owners: load, slice, deposit (as in the large tile, with 16 group words per party) ----------------
    U64x2 xa[Q::kPairs], xb[Q::kPairs];
#pragma unroll
    for (int c = 0; c < Q::kPairs; ++c) {
        const int pr = c * kWave + lane;
        const int e = 2 * pr;
        xa[c] = U64x2{0, 0};
        xb[c] = U64x2{0, 0};
        if (e < Q::kTile) {
            io.template load_pair<FULL>(tile0, (unsigned)e, n, xa[c], xb[c]);
            if constexpr (T::kPacked) {
                using Item = typename T::Item;
                Item *w0 = reinterpret_cast<Item *>(slice_lds);
                Item *w1 = reinterpret_cast<Item *>(slice_lds + Q::kGroups * 8);
                w0[pr] = (Item)(((xa[c].a >> k) & S::kField) | (((xa[c].b >> k) & S::kField) << (W % 64)));
                w1[pr] = (Item)(((xb[c].a >> k) & S::kField) | (((xb[c].b >> k) & S::kField) << (W % 64)));
            } else {
                using Entry = typename T::Entry;
                Entry *slices = reinterpret_cast<Entry *>(slice_lds);
                slices[e] = (Entry)((xa[c].a >> k) & S::kField) | ((Entry)((xb[c].a >> k) & S::kField) << T::kHalf);
                slices[e + 1] = (Entry)((xa[c].b >> k) & S::kField) | ((Entry)((xb[c].b >> k) & S::kField) << T::kHalf);
            }
        }
    }

    // ---- every lane: its share of the group's dealer words -------------------------------------------------
    const int grp = lane / Q::kSplit, sub = lane % Q::kSplit;
    const uint64_t g = tile * Q::kGroups + grp;
    const uint64_t zg = seedB + (g * (uint64_t)S::words_per_group(false) + 1) * kGamma;
    uint64_t *gw = words_lds + grp * Q::kStride;
#pragma unroll
    for (int t = 0; t < Q::kWordsPerLane; ++t) {
        const int j = t * Q::kSplit + sub;                      // j-th evaluated word: stream index j, the B2A word last
        if (Q::kWords % Q::kSplit == 0 || t + 1 < Q::kWordsPerLane || j < Q::kWords) {
            const unsigned idx = (j == Q::kWords - 1) ? (unsigned)S::b2a_word(false) : (unsigned)j;
            gw[j] = mix64(zg + (uint64_t)idx * kGamma);
        }
    }
    wave_sync();

    // ---- every lane: collect the fields of its group, run the gate logic on the exchanged words ------------
    uint64_t u0 = 0, u1 = 0;
    if constexpr (T::kPacked) {
        u0 = reinterpret_cast<const uint64_t *>(slice_lds)[grp];
        u1 = reinterpret_cast<const uint64_t *>(slice_lds + Q::kGroups * 8)[grp];
    } else {
        using Entry = typename T::Entry;
        const Entry *slices = reinterpret_cast<const Entry *>(slice_lds);
#pragma unroll
        for (int j = 0; j < L; ++j) {
            const Entry en = slices[grp * L + j];
            u0 |= (uint64_t)(en & (Entry)S::kField) << (j * W);
            u1 |= (uint64_t)(en >> T::kHalf) << (j * W);
        }
    }
    const Pair sum = a2b_sum_words<W>(u0, u1, gw);
    const uint64_t ones = S::ones();
    const uint64_t sg = ((sum.p0 >> (W - 1)) & ones) | (((sum.p1 >> (W - 1)) & ones) << T::kSign1);
    if (sub == 0) verdict[grp] = U64x2{sg, gw[Q::kWords - 1]};
    wave_sync();

    // ---- owners: pick up the verdict of each element's group, finish, store -------------------------------
    const uint64_t zA0 = seedA + (6 * (tile0 + 2 * (uint64_t)lane) + 1) * kGamma;
#pragma unroll
    for (int c = 0; c < Q::kPairs; ++c) {
        const int e = 2 * (c * kWave + lane);
        if (e < Q::kTile) {
            Pair r[2];
            const int grp0 = e / L, j0 = e - grp0 * L;
            const U64x2 v0 = verdict[grp0];
            const bool split = (L % 2 != 0) && (j0 == L - 1);
            const U64x2 v1 = split ? verdict[grp0 + 1] : v0;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const U64x2 v = h ? v1 : v0;
                const int j = h ? (split ? 0 : j0 + 1) : j0;
                const uint64_t sgj = v.a >> (j * W);
                const Pair sign{sgj & 1u, (sgj >> T::kSign1) & 1u};
                const uint32_t rh = (uint32_t)(v.b >> (2 * j));
                const Pair rho{rh & 1u, (rh >> 1) & 1u};
                const uint64_t zA = zA0 + (uint64_t)(6 * (2 * c * kWave + h)) * kGamma;
                const Pair D = b2a_drelu(sign, rho, zA);
                r[h] = (op_of(MODE) == kDrelu) ? D : beaver_mul(Pair{h ? xa[c].b : xa[c].a, h ? xb[c].b : xb[c].a}, D, zA);
            }
            io.template store_pair<FULL>(tile0, (unsigned)e, n, r[0], r[1]);
        }
    }
}

// Several tensors of one slice width on small wave-tiles; tile_end counts small tiles.
template <int W, int MODE>
__global__ void __launch_bounds__(kBlock)
small_batch_kernel(const BatchArgs args)
{
    using T = TileTraits<W>;
    using Q = SmallTraits<W>;
    __shared__ __attribute__((aligned(16))) unsigned char slices_all[kWavesPerBlock][Q::kSliceBytes];
    __shared__ __attribute__((aligned(16))) uint64_t words_all[kWavesPerBlock][Q::kGroups * Q::kStride];
    __shared__ U64x2 verdict_all[kWavesPerBlock][Q::kGroups + 1];
    const int lane = threadIdx.x % kWave, wv = wave_index();
    const uint64_t gt = (uint64_t)blockIdx.x * kWavesPerBlock + wv;
    if (gt >= args.tile_end[args.count - 1]) return;
    int ti = 0;
    while (gt >= args.tile_end[ti]) ++ti;
    const uint64_t tile = gt - (ti ? args.tile_end[ti - 1] : 0);
    const BatchTensor &d = args.t[ti];
    const ShareIO io{d.x0, d.x1, d.o0, d.o1};
    if ((tile + 1) * Q::kTile <= d.n)
        small_tile_body_impl<W, MODE, true>(io, d.n, d.k, d.seedB, d.seedA, tile, lane, slices_all[wv], words_all[wv], verdict_all[wv]);
    else
        small_tile_body_impl<W, MODE, false>(io, d.n, d.k, d.seedB, d.seedA, tile, lane, slices_all[wv], words_all[wv], verdict_all[wv]);
    (void)sizeof(T);
}

// The simulator kernel: ReLU on plaintext floats through the whole protocol, 8 bytes of traffic per element.
// Slice widths up to 32 run the wave-tile body; wider slices (one element per word) take one thread per element.
template <int W>
__global__ void __launch_bounds__(kBlock)
wide_sim_kernel(const float *x, uint64_t n, int k, uint64_t seedB, uint64_t seedA, uint64_t seedS, float *y)
{
    using S = Shape<W>;
    static_assert(S::L == 1, "one element per word");
    const uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n) return;
    const uint64_t x0 = mix64(seedS + (i + 1) * kGamma);
    const uint64_t x1 = encode_fixed16(x[i]) - x0;
    const uint64_t zg = seedB + (i * (uint64_t)S::words_per_group(false) + 1) * kGamma;
    const Pair sum = a2b_sum<W, false>((x0 >> k) & S::kField, (x1 >> k) & S::kField, zg);
    const uint64_t wb = mix64(zg + (uint64_t)S::b2a_word(false) * kGamma);
    const Pair r = finish_element<W, kRelu>(sum, wb, 0, Pair{x0, x1}, seedA + (6 * i + 1) * kGamma);
    y[i] = decode_fixed16(r.p0 + r.p1);
}

template <int W>
__global__ void __launch_bounds__(kBlock)
tile_sim_kernel(const float *x, uint64_t n, int k, uint64_t seedB, uint64_t seedA, uint64_t seedS, float *y)
{
    using T = TileTraits<W>;
    __shared__ __attribute__((aligned(16))) unsigned char slices_all[kWavesPerBlock][T::kSliceBytes];
    __shared__ U64x2 verdict_all[kWavesPerBlock][kWave];
    const int lane = threadIdx.x % kWave, wv = wave_index();
    const uint64_t tile = (uint64_t)blockIdx.x * kWavesPerBlock + wv;
    if (tile * T::kTile >= n) return;
    tile_body<W, kRelu>(FloatIO{x, y, seedS}, n, k, seedB, seedA, tile, lane, slices_all[wv], verdict_all[wv]);
}

}  // namespace hb
