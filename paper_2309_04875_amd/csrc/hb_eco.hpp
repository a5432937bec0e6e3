// Zero-error high-cut scan (paper Sec. 4.1.2, the "eco" strategy: keep bits [0, m) with the smallest m
// that changes no DReLU result).  With no low cut the two slices are exact shares of x mod 2^m
// (Theorem 1's proof), so DReLU on [0, m) is 1 - bit_{m-1}(x) and it differs from the full-ring result
// exactly when bit m-1 of x differs from its sign bit.  Per element that is one 64-bit word
// d = x ^ (x >>arith 63), and counts[m-1] is the number of elements with bit m-1 of d set.
//
// The 64 population counts are taken without ever touching a counter per element: every lane keeps a
// bit-sliced counter (plane j holds bit j of all 64 per-position counts) and feeds it through a
// carry-save adder tree, two v_bitop3_b32 per 64-bit carry-save step.  The kernel streams 16 bytes per
// element and is bound by HBM.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hb_kernels.hpp"

namespace hb {

constexpr int kEcoPlanes = 16;          // a lane may count up to 2^16 - 1 elements
constexpr int kEcoChunk = 64;           // elements per lane consumed by one carry-save tree
constexpr int kEcoMaxPerLane = 32768;

__device__ __forceinline__ uint64_t bit3(uint64_t a, uint64_t b, uint64_t c, bool majority)
{
    // xor3: 0xF0 ^ 0xCC ^ 0xAA = 0x96; majority: (a&b)|(a&c)|(b&c) = 0xE8
    uint32_t lo, hi;
    if (majority) {
        lo = __builtin_amdgcn_bitop3_b32((uint32_t)a, (uint32_t)b, (uint32_t)c, 0xE8);
        hi = __builtin_amdgcn_bitop3_b32((uint32_t)(a >> 32), (uint32_t)(b >> 32), (uint32_t)(c >> 32), 0xE8);
    } else {
        lo = __builtin_amdgcn_bitop3_b32((uint32_t)a, (uint32_t)b, (uint32_t)c, 0x96);
        hi = __builtin_amdgcn_bitop3_b32((uint32_t)(a >> 32), (uint32_t)(b >> 32), (uint32_t)(c >> 32), 0x96);
    }
    return ((uint64_t)hi << 32) | lo;
}

template <bool VEC>
struct EcoLoader {
    const uint64_t *x0, *x1;
    uint64_t n;
    uint64_t base;      // first element of this lane's current chunk row: element(idx) = base + (idx/2)*128 + idx%2
    // word idx (0..63) of the lane's chunk: sign-disagreement word of one element
    __device__ __forceinline__ void load_pair(int pair, uint64_t &d0, uint64_t &d1) const
    {
        const uint64_t i = base + (uint64_t)pair * (2 * kWave);
        uint64_t a0 = 0, a1 = 0, b0 = 0, b1 = 0;
        if (i + 1 < n) {
            if (VEC) {
                const U64x2 a = load_stream2(x0 + i);
                const U64x2 b = load_stream2(x1 + i);
                a0 = a.a; a1 = a.b; b0 = b.a; b1 = b.b;
            } else {
                a0 = load_stream(x0 + i); a1 = load_stream(x0 + i + 1); b0 = load_stream(x1 + i); b1 = load_stream(x1 + i + 1);
            }
        } else if (i < n) {
            a0 = load_stream(x0 + i);
            b0 = load_stream(x1 + i);
        }
        const uint64_t xa = a0 + b0, xb = a1 + b1;
        d0 = xa ^ (uint64_t)((int64_t)xa >> 63);
        d1 = xb ^ (uint64_t)((int64_t)xb >> 63);
    }
};

// Word of weight 2^J summarising 2^J consecutive inputs starting at input idx * 2^J; planes 0..J-1 absorb the rest.
template <int J, class Loader>
__device__ __forceinline__ uint64_t eco_level(uint64_t (&plane)[kEcoPlanes], const Loader &ld, int idx)
{
    if constexpr (J == 1) {
        uint64_t d0, d1;
        ld.load_pair(idx, d0, d1);
        const uint64_t carry = bit3(plane[0], d0, d1, true);
        plane[0] = bit3(plane[0], d0, d1, false);
        return carry;
    } else {
        const uint64_t a = eco_level<J - 1, Loader>(plane, ld, 2 * idx);
        const uint64_t b = eco_level<J - 1, Loader>(plane, ld, 2 * idx + 1);
        const uint64_t carry = bit3(plane[J - 1], a, b, true);
        plane[J - 1] = bit3(plane[J - 1], a, b, false);
        return carry;
    }
}

__global__ void __launch_bounds__(64) eco_zero_kernel(unsigned long long *counts) { counts[threadIdx.x] = 0; }

// chunks: number of 64-element chunks each lane consumes; a wavefront covers 64 * 64 * chunks consecutive elements.
template <bool VEC>
__global__ void __launch_bounds__(kBlock)
eco_scan_kernel(const uint64_t *x0, const uint64_t *x1, uint64_t n, int chunks, int live_planes, unsigned long long *counts)
{
    __shared__ unsigned int partial[kWavesPerBlock][64];
    const int lane = threadIdx.x % kWave, wv = threadIdx.x / kWave;
    const uint64_t wave = (uint64_t)blockIdx.x * kWavesPerBlock + wv;
    const uint64_t per_wave = (uint64_t)kWave * kEcoChunk * (uint64_t)chunks;

    uint64_t plane[kEcoPlanes];
#pragma unroll
    for (int j = 0; j < kEcoPlanes; ++j) plane[j] = 0;

    EcoLoader<VEC> ld{x0, x1, n, 0};
    for (int c = 0; c < chunks; ++c) {
        ld.base = wave * per_wave + (uint64_t)c * (kWave * kEcoChunk) + 2 * (uint64_t)lane;
        if (ld.base - 2 * (uint64_t)lane >= n) break;                 // uniform per wave
        uint64_t carry = eco_level<6, EcoLoader<VEC>>(plane, ld, 0);                  // 64 elements -> planes 0..5 + a weight-64 word
#pragma unroll
        for (int j = 6; j < kEcoPlanes; ++j) {                        // ripple the carry into the upper planes
            const uint64_t t = plane[j] & carry;
            plane[j] ^= carry;
            carry = t;
        }
    }

    // Per-position totals of the wavefront.  The 64 lanes' bit-sliced counters are summed by a butterfly of six
    // bit-sliced additions (lane l with lane l ^ 32, ^ 16, ... ^ 1; a full adder per plane is two v_bitop3_b32 per
    // half), after which every lane holds the wavefront's totals, still bit-sliced: up to 16 + 6 planes.  Lane b
    // then reads position b out of every plane.
    uint64_t tot[kEcoPlanes + 6];
#pragma unroll
    for (int j = 0; j < kEcoPlanes + 6; ++j) tot[j] = j < kEcoPlanes ? plane[j] : 0;
#pragma unroll
    for (int level = 0; level < 6; ++level) {
        const int stride = 32 >> level;
        uint64_t carry = 0;
#pragma unroll
        for (int j = 0; j < kEcoPlanes + 6; ++j) {
            if (j < live_planes + level) {                            // planes above are still zero (uniform)
                const uint32_t lo = __shfl_xor((uint32_t)tot[j], stride, kWave);
                const uint32_t hi = __shfl_xor((uint32_t)(tot[j] >> 32), stride, kWave);
                const uint64_t other = ((uint64_t)hi << 32) | lo;
                const uint64_t sum = bit3(tot[j], other, carry, false);
                carry = bit3(tot[j], other, carry, true);
                tot[j] = sum;
            } else if (j == live_planes + level) {
                tot[j] = carry;                                       // the sum is one plane longer
            }
        }
    }
    unsigned int mine = 0;                                            // lane b: the total for position b
#pragma unroll
    for (int j = 0; j < kEcoPlanes + 6; ++j) {
        if (j < live_planes + 6) mine |= (unsigned int)((tot[j] >> lane) & 1) << j;
    }
    partial[wv][lane] = mine;
    __syncthreads();
    if (wv == 0) {
        unsigned long long sum = 0;
#pragma unroll
        for (int v = 0; v < kWavesPerBlock; ++v) sum += partial[v][lane];
        if (sum != 0) atomicAdd(&counts[lane], sum);
    }
}

}  // namespace hb
