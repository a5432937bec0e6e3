// Instantiates the multi-party kernels of one party count for slice widths HB_PART_LO..HB_PART_HI (DReLU and
// ReLU) and registers their launchers.  Compiled several times with different -D values so the parts build in
// parallel.
#include "hb_launch.hpp"
#include "hb_multiparty.hpp"

#if !defined(HB_PART_PARTIES) || !defined(HB_PART_LO) || !defined(HB_PART_HI)
#error "compile with -DHB_PART_PARTIES=<3|4> -DHB_PART_LO=<w> -DHB_PART_HI=<w>"
#endif

namespace {

template <int W, int P, int MODE>
hipError_t launch_mp(const hb::MpPointers &ptr, uint64_t n, int k, uint64_t seedB, uint64_t seedA, hipStream_t stream)
{
    if constexpr (hb::MpTileTraits<W, P>::kSupported) {
        if (!hb::force_group_kernel()) {
            const uint64_t wave_tiles = (n + hb::MpTileTraits<W, P>::kTile - 1) / hb::MpTileTraits<W, P>::kTile;
            const uint64_t blocks = (wave_tiles + hb::kWavesPerBlock - 1) / hb::kWavesPerBlock;
            if (blocks == 0 || blocks > 0x7fffffffull) return hipErrorInvalidConfiguration;
            hipLaunchKernelGGL((hb::mp_tile_kernel<W, P, MODE>), dim3((unsigned)blocks), dim3(hb::kBlock), 0, stream, ptr,
                               n, k, seedB, seedA);
            return hipGetLastError();
        }
    }
    constexpr uint64_t L = hb::MpShape<W, P>::L;
    const uint64_t groups = (n + L - 1) / L;
    const uint64_t blocks = (groups + hb::kBlock - 1) / hb::kBlock;
    if (blocks == 0 || blocks > 0x7fffffffull) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((hb::mp_group_kernel<W, P, MODE>), dim3((unsigned)blocks), dim3(hb::kBlock), 0, stream, ptr, n,
                       groups, k, seedB, seedA);
    return hipGetLastError();
}

template <int W>
void fill(hb::LauncherTable &t)
{
    t.mp[HB_PART_PARTIES - 3][hb::kDrelu][W - 1] = &launch_mp<W, HB_PART_PARTIES, hb::kDrelu>;
    t.mp[HB_PART_PARTIES - 3][hb::kRelu][W - 1] = &launch_mp<W, HB_PART_PARTIES, hb::kRelu>;
    if constexpr (W < HB_PART_HI) fill<W + 1>(t);
}

struct Registrar {
    Registrar() { fill<HB_PART_LO>(hb::launcher_table()); }
};
const Registrar g_registrar;

}  // namespace
