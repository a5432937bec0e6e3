// Float boundary of the simulator (paper Sec. 4.1.1: convert floating point values to ring elements, generate
// secret shares, ... ): stand-alone encode-and-share and open-and-decode kernels.  Included by one translation unit.
#pragma once

#include "hb_kernels.hpp"

namespace hb {

// Encode and share: share0[i] = output i of the stream started at seedS, share1[i] = round(2^16 x[i]) - share0[i].
__global__ void __launch_bounds__(kBlock)
share_f32_kernel(const float *x, uint64_t n, uint64_t seedS, uint64_t *s0, uint64_t *s1)
{
    const uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n) return;
    const uint64_t r = mix64(seedS + (i + 1) * kGamma);
    s0[i] = r;
    s1[i] = encode_fixed16(x[i]) - r;
}

// Open and decode: y[i] = (share0[i] + share1[i]) / 2^16 as a float.
__global__ void __launch_bounds__(kBlock)
reveal_f32_kernel(const uint64_t *s0, const uint64_t *s1, uint64_t n, float *y)
{
    const uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n) return;
    y[i] = decode_fixed16(s0[i] + s1[i]);
}

}  // namespace hb
