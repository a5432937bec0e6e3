// Instantiates the group kernels of one mode for slice widths HB_PART_LO..HB_PART_HI and registers
// their launchers.  Compiled several times with different -D values so the parts build in parallel.
#include "hb_kernels.hpp"
#include "hb_launch.hpp"

#if !defined(HB_PART_MODE) || !defined(HB_PART_LO) || !defined(HB_PART_HI)
#error "compile with -DHB_PART_MODE=<0..4> -DHB_PART_LO=<w> -DHB_PART_HI=<w>"
#endif

namespace {

template <int W, int MODE>
hipError_t launch_group(const uint64_t *x0, const uint64_t *x1, uint64_t n, int k, uint64_t seedB, uint64_t seedA,
                        uint64_t *o0, uint64_t *o1, bool vec16, hipStream_t stream)
{
    constexpr uint64_t L = hb::Shape<W>::L;
    const uint64_t groups = (n + L - 1) / L;
    const uint64_t blocks = (groups + hb::kBlock - 1) / hb::kBlock;
    if (blocks == 0 || blocks > 0x7fffffffull) return hipErrorInvalidConfiguration;
    if constexpr (hb::TileTraits<W>::kSupported) {
        if (!hb::force_group_kernel()) {
            const uint64_t wave_tiles = (n + hb::TileTraits<W>::kTile - 1) / hb::TileTraits<W>::kTile;
            const uint64_t tiles = (wave_tiles + hb::kWavesPerBlock - 1) / hb::kWavesPerBlock;
            if (tiles > 0x7fffffffull) return hipErrorInvalidConfiguration;
            hipLaunchKernelGGL((hb::tile_kernel<W, MODE>), dim3((unsigned)tiles), dim3(hb::kBlock), 0, stream, x0, x1, n, k,
                               seedB, seedA, o0, o1);
            return hipGetLastError();
        }
    }
    if (vec16) {
        hipLaunchKernelGGL((hb::group_kernel<W, MODE, true>), dim3((unsigned)blocks), dim3(hb::kBlock), 0, stream, x0,
                           x1, n, groups, k, seedB, seedA, o0, o1);
    } else {
        hipLaunchKernelGGL((hb::group_kernel<W, MODE, false>), dim3((unsigned)blocks), dim3(hb::kBlock), 0, stream, x0,
                           x1, n, groups, k, seedB, seedA, o0, o1);
    }
    return hipGetLastError();
}

template <int W, int MODE>
hipError_t launch_batch(const hb::BatchArgs &args, hipStream_t stream)
{
    if constexpr (hb::TileTraits<W>::kSupported) {
        const uint64_t wave_tiles = args.tile_end[args.count - 1];
        const uint64_t blocks = (wave_tiles + hb::kWavesPerBlock - 1) / hb::kWavesPerBlock;
        if (blocks == 0 || blocks > 0x7fffffffull) return hipErrorInvalidConfiguration;
        hipLaunchKernelGGL((hb::tile_batch_kernel<W, MODE>), dim3((unsigned)blocks), dim3(hb::kBlock), 0, stream, args);
        return hipGetLastError();
    } else {
        return hipErrorInvalidDeviceFunction;
    }
}

constexpr bool kSmallMode = (HB_PART_MODE == hb::kDrelu || HB_PART_MODE == hb::kRelu);

template <int W, int MODE>
hipError_t launch_small_batch(const hb::BatchArgs &args, hipStream_t stream)
{
    if constexpr (hb::SmallTraits<W>::kSupported && kSmallMode) {
        const uint64_t wave_tiles = args.tile_end[args.count - 1];
        const uint64_t blocks = (wave_tiles + hb::kWavesPerBlock - 1) / hb::kWavesPerBlock;
        if (blocks == 0 || blocks > 0x7fffffffull) return hipErrorInvalidConfiguration;
        hipLaunchKernelGGL((hb::small_batch_kernel<W, MODE>), dim3((unsigned)blocks), dim3(hb::kBlock), 0, stream, args);
        return hipGetLastError();
    } else {
        return hipErrorInvalidDeviceFunction;
    }
}

template <int W>
hipError_t launch_sim(const float *x, uint64_t n, int k, uint64_t seedB, uint64_t seedA, uint64_t seedS, float *y,
                      hipStream_t stream)
{
    if constexpr (HB_PART_MODE != hb::kRelu) {
        return hipErrorInvalidDeviceFunction;
    } else if constexpr (hb::TileTraits<W>::kSupported) {
        const uint64_t wave_tiles = (n + hb::TileTraits<W>::kTile - 1) / hb::TileTraits<W>::kTile;
        const uint64_t blocks = (wave_tiles + hb::kWavesPerBlock - 1) / hb::kWavesPerBlock;
        if (blocks == 0 || blocks > 0x7fffffffull) return hipErrorInvalidConfiguration;
        hipLaunchKernelGGL((hb::tile_sim_kernel<W>), dim3((unsigned)blocks), dim3(hb::kBlock), 0, stream, x, n, k, seedB,
                           seedA, seedS, y);
        return hipGetLastError();
    } else {
        const uint64_t blocks = (n + hb::kBlock - 1) / hb::kBlock;
        if (blocks == 0 || blocks > 0x7fffffffull) return hipErrorInvalidConfiguration;
        hipLaunchKernelGGL((hb::wide_sim_kernel<W>), dim3((unsigned)blocks), dim3(hb::kBlock), 0, stream, x, n, k, seedB,
                           seedA, seedS, y);
        return hipGetLastError();
    }
}

template <int W>
void fill(hb::LauncherTable &t)
{
    if (HB_PART_MODE == hb::kRelu) t.sim[W - 1] = &launch_sim<W>;
    t.f[HB_PART_MODE][W - 1] = &launch_group<W, HB_PART_MODE>;
    t.batch[HB_PART_MODE][W - 1] = hb::TileTraits<W>::kSupported ? &launch_batch<W, HB_PART_MODE> : nullptr;
    t.small[HB_PART_MODE][W - 1] = (hb::SmallTraits<W>::kSupported && kSmallMode) ? &launch_small_batch<W, HB_PART_MODE> : nullptr;
    if constexpr (W < HB_PART_HI) fill<W + 1>(t);
}

struct Registrar {
    Registrar() { fill<HB_PART_LO>(hb::launcher_table()); }
};
const Registrar g_registrar;

}  // namespace
