// Kernels: one thread evaluates one group of L = min(64/W, 32) consecutive elements.
//
// A thread packs the slices of its L elements of both shares into two SWAR words, runs the whole
// circuit on them in registers (gate 0, all prefix rounds, sign), then finishes its elements one by
// one (B2A, Beaver multiply) and stores the result shares.  Nothing but the input shares is read from
// memory and nothing but the output shares is written: the algorithmic traffic is 32 bytes per element.
#pragma once

#include "hb_protocol.hpp"

namespace hb {

constexpr int kBlock = 256;

struct alignas(16) U64x2 {
    uint64_t a, b;
};

template <int W, int MODE, bool VEC>
__global__ void __launch_bounds__(kBlock)
group_kernel(const uint64_t *x0, const uint64_t *x1, uint64_t n, uint64_t groups, int k, uint64_t seedB,
             uint64_t seedA, uint64_t *o0, uint64_t *o1)
{
    using S = Shape<W>;
    constexpr int L = S::L;
    // keep the loaded shares in registers across the circuit when that is cheap, else read them again
    constexpr bool kHold = (MODE == kRelu) && (L <= 8);

    const uint64_t g = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (g >= groups) return;
    const uint64_t i0 = g * (uint64_t)L;
    const bool full = (n - i0) >= (uint64_t)L;
    const int cnt = full ? L : (int)(n - i0);

    uint64_t xa[kHold ? L : 1], xb[kHold ? L : 1];
    uint64_t u0 = 0, u1 = 0;

    if (VEC && full && (L % 2 == 0)) {
        const U64x2 *v0 = reinterpret_cast<const U64x2 *>(x0 + i0);
        const U64x2 *v1 = reinterpret_cast<const U64x2 *>(x1 + i0);
#pragma unroll
        for (int j = 0; j < L / 2; ++j) {
            const U64x2 a = v0[j], b = v1[j];
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
                a = x0[i0 + j];
                b = x1[i0 + j];
            }
            u0 |= ((a >> k) & S::kField) << (j * W % 64);
            u1 |= ((b >> k) & S::kField) << (j * W % 64);
            if (kHold) {
                xa[j] = a;
                xb[j] = b;
            }
        }
    }

    const uint64_t zg = seedB + (g * (uint64_t)S::kWordsPerGroup + 1) * kGamma;
    const Pair sum = a2b_sum<W>(u0, u1, zg);
    uint64_t wb = 0;
    if (MODE != kSign) wb = mix64(zg + (uint64_t)(5 * S::kGates) * kGamma);

    const uint64_t zA0 = seedA + (6 * i0 + 1) * kGamma;
    if (VEC && full && (L % 2 == 0)) {
        U64x2 *w0 = reinterpret_cast<U64x2 *>(o0 + i0);
        U64x2 *w1 = reinterpret_cast<U64x2 *>(o1 + i0);
#pragma unroll
        for (int j = 0; j < L / 2; ++j) {
            Pair xe{0, 0}, xo{0, 0};
            if (MODE == kRelu) {
                if (kHold) {
                    xe = Pair{xa[2 * j], xb[2 * j]};
                    xo = Pair{xa[2 * j + 1], xb[2 * j + 1]};
                } else {
                    const U64x2 a = reinterpret_cast<const U64x2 *>(x0 + i0)[j];
                    const U64x2 b = reinterpret_cast<const U64x2 *>(x1 + i0)[j];
                    xe = Pair{a.a, b.a};
                    xo = Pair{a.b, b.b};
                }
            }
            const Pair re = finish_element<W, MODE>(sum, wb, 2 * j, xe, zA0 + (uint64_t)(6 * (2 * j)) * kGamma);
            const Pair ro = finish_element<W, MODE>(sum, wb, 2 * j + 1, xo, zA0 + (uint64_t)(6 * (2 * j + 1)) * kGamma);
            w0[j] = U64x2{re.p0, ro.p0};
            w1[j] = U64x2{re.p1, ro.p1};
        }
    } else {
#pragma unroll
        for (int j = 0; j < L; ++j) {
            if (j < cnt) {
                Pair x{0, 0};
                if (MODE == kRelu) x = kHold ? Pair{xa[j], xb[j]} : Pair{x0[i0 + j], x1[i0 + j]};
                const Pair r = finish_element<W, MODE>(sum, wb, j, x, zA0 + (uint64_t)(6 * j) * kGamma);
                o0[i0 + j] = r.p0;
                o1[i0 + j] = r.p1;
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
            const U64x2 a = reinterpret_cast<const U64x2 *>(x0)[t];
            const U64x2 b = reinterpret_cast<const U64x2 *>(x1)[t];
            reinterpret_cast<U64x2 *>(out)[t] = binary ? U64x2{a.a ^ b.a, a.b ^ b.b} : U64x2{a.a + b.a, a.b + b.b};
        } else if (i < n) {
            out[i] = binary ? (x0[i] ^ x1[i]) : (x0[i] + x1[i]);
        }
    } else {
        if (t < n) out[t] = binary ? (x0[t] ^ x1[t]) : (x0[t] + x1[t]);
    }
}

}  // namespace hb
