// Compile-only probe: one kernel per (slice width, mode) that runs the bounds-check-free tile body once, so that
// the SplitMix64 evaluations in its machine code can be counted (tests/test_kernel_dealer_words.py).
#include "hb_multiparty.hpp"

using namespace hb;

template <int W, int MODE>
__device__ __forceinline__ void probe_body(const uint64_t *x0, const uint64_t *x1, uint64_t n, int k, uint64_t seedB,
                                           uint64_t seedA, uint64_t *o0, uint64_t *o1)
{
    using T = TileTraits<W>;
    __shared__ __attribute__((aligned(16))) unsigned char slices_all[kWavesPerBlock][T::kSliceBytes];
    __shared__ U64x2 verdict_all[kWavesPerBlock][kWave];
    const int lane = threadIdx.x % kWave, wv = wave_index();
    const uint64_t tile = (uint64_t)blockIdx.x * kWavesPerBlock + wv;
    tile_body_impl<W, MODE, true>(ShareIO{x0, x1, o0, o1}, n, k, seedB, seedA, tile, lane, slices_all[wv], verdict_all[wv]);
}

#define PROBE(NAME, W, MODE)                                                                                        \
    extern "C" __global__ void __launch_bounds__(kBlock) NAME(const uint64_t *x0, const uint64_t *x1, uint64_t n,    \
                                                              int k, uint64_t seedB, uint64_t seedA, uint64_t *o0,   \
                                                              uint64_t *o1)                                          \
    {                                                                                                               \
        probe_body<W, MODE>(x0, x1, n, k, seedB, seedA, o0, o1);                                                    \
    }

PROBE(probe_w8_relu, 8, kRelu)
PROBE(probe_w8_drelu, 8, kDrelu)
PROBE(probe_w8_relu_shared, 8, kReluShared)
PROBE(probe_w16_relu, 16, kRelu)
PROBE(probe_w6_relu, 6, kRelu)

// the same for the multi-party tile body
template <int W, int P, int MODE>
__device__ __forceinline__ void mp_probe_body(const MpPointers &ptr, uint64_t n, int k, uint64_t seedB, uint64_t seedA)
{
    using T = MpTileTraits<W, P>;
    __shared__ __attribute__((aligned(16))) unsigned char slices_all[kWavesPerBlock][P][T::kSliceBytes];
    __shared__ U64x2 verdict_all[kWavesPerBlock][kWave];
    const int lane = threadIdx.x % kWave, wv = wave_index();
    const uint64_t tile = (uint64_t)blockIdx.x * kWavesPerBlock + wv;
    mp_tile_body<W, P, MODE, true>(ptr, n, k, seedB, seedA, tile, lane, slices_all[wv], verdict_all[wv]);
}

#define MP_PROBE(NAME, W, P, MODE)                                                                                  \
    extern "C" __global__ void __launch_bounds__(kBlock) NAME(const MpPointers ptr, uint64_t n, int k, uint64_t seedB, \
                                                              uint64_t seedA)                                        \
    {                                                                                                               \
        mp_probe_body<W, P, MODE>(ptr, n, k, seedB, seedA);                                                          \
    }

MP_PROBE(probe_p3_w8_relu, 8, 3, kRelu)
MP_PROBE(probe_p3_w8_drelu, 8, 3, kDrelu)
MP_PROBE(probe_p4_w8_relu, 8, 4, kRelu)
