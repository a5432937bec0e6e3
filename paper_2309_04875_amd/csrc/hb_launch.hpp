// Table of kernel launchers indexed by (mode, slice width).  The kernels are instantiated in several
// translation units (hb_launch_part.hip compiled once per mode and width range) that register
// themselves here when the library is loaded.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hb_kernels.hpp"
#include "hb_multiparty.hpp"

namespace hb {

using GroupLauncher = hipError_t (*)(const uint64_t *x0, const uint64_t *x1, uint64_t n, int k, uint64_t seedB,
                                     uint64_t seedA, uint64_t *o0, uint64_t *o1, bool vec16, hipStream_t stream);

// Launches the tensors described by `args` (all of one slice width, tile-kernel eligible) in one grid.
using BatchLauncher = hipError_t (*)(const BatchArgs &args, hipStream_t stream);

// The float-in / float-out simulator kernel of one slice width.
using SimLauncher = hipError_t (*)(const float *x, uint64_t n, int k, uint64_t seedB, uint64_t seedA, uint64_t seedS,
                                   float *y, hipStream_t stream);

// DReLU / ReLU among 3 or 4 parties.
using MpLauncher = hipError_t (*)(const MpPointers &ptr, uint64_t n, int k, uint64_t seedB, uint64_t seedA,
                                  hipStream_t stream);

struct LauncherTable {
    GroupLauncher f[kModes][64];       // [mode][w - 1]
    BatchLauncher batch[kModes][64];   // null where the width has no tile kernel
    BatchLauncher small[kModes][64];   // small wave-tiles (tile_end counts small tiles); null where there is none
    SimLauncher sim[64];               // null where the width has no tile kernel
    MpLauncher mp[kMaxParties - 2][2][64];   // [parties - 3][kDrelu | kRelu][w - 1]
};

LauncherTable &launcher_table();

// Debug knob: HB_KERNEL=group in the environment (read once) sends every width to the thread-per-group kernel.
bool force_group_kernel();

}  // namespace hb
